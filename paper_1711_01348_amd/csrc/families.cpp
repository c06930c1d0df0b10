// Pattern recognition: which kernel family evaluates the forward pass and each gradient.
// Every plan can run on the plan-driven generic kernels; a specialised family is chosen only
// when body, index matrices, shapes and dtype match its template exactly, and the derived plan
// has the structure the family's kernels assume (which kernel coordinate collapses, which is a window).
#include <algorithm>

#include "plan.hpp"
#include "launch_geom.h"

namespace tad {

// 24-bit safety of the loop-free form: every coefficient and every index extent below 2^23
static bool fits24(int64_t v) { return v > -(1 << 23) && v < (1 << 23); }
static bool extents_fit24(const GatherPlan &g) {
    for (int r = 0; r < g.rank; ++r)
        if (!fits24(g.shape[r])) return false;
    return true;
}

// Largest |y_c| a kernel can meet for gradient elements inside the shape: y = (U beta) / alpha.
static int64_t y_extent(const GatherPlan &g, int c) {
    int64_t v = 0;
    for (int d = 0; d < g.rank; ++d) v += (g.U[c][d] < 0 ? -(int64_t)g.U[c][d] : g.U[c][d]) * (g.shape[d] - 1);
    return v;   // dividing by alpha_c >= 1 only makes it smaller
}

bool flatten_level(const GatherPlan &g, int level, FlatLevel &out) {
    if (level < 0 || level >= g.kappa || g.R > kFlatY || !extents_fit24(g)) return false;
    const int nl = g.lo_end[level] - g.lo_begin[level], nh = g.hi_end[level] - g.hi_begin[level];
    if (nl > kFlatRows || nh > kFlatRows) return false;
    for (int r = 0; r < kFlatRows; ++r) {
        out.ls[r] = 1; out.lk0[r] = kFlatNeutralLo;   // neutral lower row
        out.hs[r] = 1; out.hk0[r] = kFlatNeutralHi;   // neutral upper row
        out.lrs[r] = out.hrs[r] = 1.f;
        for (int c = 0; c < kFlatY; ++c) out.lky[r][c] = out.hky[r][c] = 0;
    }
    for (int r = 0; r < nl + nh; ++r) {
        const GRow &row = g.rows[(r < nl ? g.lo_begin[level] : g.hi_begin[level] - nl) + r];
        for (int m = 0; m < kMaxKernel; ++m)
            if (row.kz[m] != 0) return false;
        for (int c = 0; c < g.R; ++c)
            if (!fits24(row.ky[c])) return false;
        // the loop-free division needs |k0 + ky . y| < 2^23 for every y the kernels can meet
        int64_t worst = row.k0 < 0 ? -(int64_t)row.k0 : row.k0;
        for (int c = 0; c < g.R; ++c) worst += (row.ky[c] < 0 ? -(int64_t)row.ky[c] : row.ky[c]) * y_extent(g, c);
        if (worst >= kFlatNeutralHi || !fits24(row.scale)) return false;
        if (r < nl) {
            out.ls[r] = row.scale; out.lk0[r] = row.k0; out.lrs[r] = 1.f / (float)row.scale;
            for (int c = 0; c < g.R; ++c) out.lky[r][c] = row.ky[c];
        } else {
            out.hs[r - nl] = row.scale; out.hk0[r - nl] = row.k0; out.hrs[r - nl] = 1.f / (float)row.scale;
            for (int c = 0; c < g.R; ++c) out.hky[r - nl][c] = row.ky[c];
        }
    }
    return true;
}

bool flatten_feas(const GatherPlan &g, FlatFeas &out) {
    if (g.nF > kFlatFeas || g.R > kFlatY || !extents_fit24(g)) return false;
    for (int r = 0; r < g.nF; ++r)
        for (int c = 0; c < g.R; ++c)
            if (!fits24(g.feas[r].ky[c])) return false;
    for (int r = 0; r < kFlatFeas; ++r) {
        out.k0[r] = -1;                               // neutral: always satisfied
        for (int c = 0; c < kFlatY; ++c) out.ky[r][c] = 0;
    }
    for (int r = 0; r < g.nF; ++r) {
        out.k0[r] = g.feas[r].k0;
        for (int c = 0; c < g.R; ++c) out.ky[r][c] = g.feas[r].ky[c];
    }
    return true;
}

bool y_is_beta(const GatherPlan &g) {
    if (g.nC != 0 || g.R != g.rank) return false;
    for (int r = 0; r < g.R; ++r) {
        if (g.diag[r] != 1) return false;
        for (int c = 0; c < g.rank; ++c)
            if (g.U[r][c] != (r == c ? 1 : 0)) return false;
    }
    return true;
}

static bool index_is(const tad_arg &a, int n_ext, std::initializer_list<std::initializer_list<int64_t>> m) {
    if ((size_t)a.rank != m.size()) return false;
    int r = 0;
    for (const auto &row : m) {
        if ((int)row.size() != n_ext) return false;
        int d = 0;
        for (int64_t v : row)
            if (a.index[r][d++] != v) return false;
        ++r;
    }
    return true;
}

static bool all_derived(const tad_plan &pl) {
    for (const auto &ap : pl.ap)
        if (!ap.derived) return false;
    return true;
}

// f_ij = exp(-sum_k((a_ik + b_jk)^2 c_ii + d_{i+k}^3)), extended index (i, j, k)
static bool match_worked(tad_plan &pl) {
    const tad_expr &e = pl.expr;
    if (e.body != TAD_BODY_WORKED || pl.dtype != TAD_F32 || e.n_f != 2 || e.n_sum != 1) return false;
    if (e.sum_lo[0] != 0 || !all_derived(pl)) return false;
    const int64_t I = e.f_shape[0], J = e.f_shape[1], K = e.sum_hi[0] + 1;
    const tad_arg &a = pl.args[0], &b = pl.args[1], &c = pl.args[2], &d = pl.args[3];
    if (!index_is(a, 3, {{1, 0, 0}, {0, 0, 1}}) || a.shape[0] != I || a.shape[1] != K) return false;
    if (!index_is(b, 3, {{0, 1, 0}, {0, 0, 1}}) || b.shape[0] != J || b.shape[1] != K) return false;
    if (!index_is(c, 3, {{1, 0, 0}, {1, 0, 0}})) return false;
    if (!index_is(d, 3, {{1, 0, 1}})) return false;
    if (J % 4 != 0) return false;   // rows of f must start 16-byte aligned for the vector loads and stores
    // plan of d: one kernel coordinate must be the collapsed j, the other the clipped window moving i
    const ArgPlan &pd = pl.ap[3];
    if (pd.smith.R != 1 || pd.K.cols != 2 || pd.VR(1, 0) != 0) return false;
    int lvl_j = -1, lvl_w = -1;
    for (int m = 0; m < 2; ++m) {
        if (pd.K(0, m) == 0 && pd.K(1, m) == 1 && pd.K(2, m) == 0) lvl_j = m;
        else if (pd.K(1, m) == 0 && pd.K(0, m) != 0) lvl_w = m;
    }
    if (lvl_j < 0 || lvl_w < 0) return false;
    if (!y_is_beta(pd.dev) || !flatten_feas(pd.dev, pl.fast.feas) || !flatten_level(pd.dev, lvl_w, pl.fast.flat[0]))
        return false;
    pl.fast.I = I; pl.fast.J = J; pl.fast.K = K;
    pl.fast.c_ld = c.shape[1];
    pl.fast.dd_level = lvl_w;
    pl.fast.dd_iy = (int)pd.VR(0, 0);
    pl.fast.dd_iz = (int)pd.K(0, lvl_w);
    if (K <= kWorkedMaxK) {
        pl.fwd_family = TAD_FAMILY_WORKED;
        for (auto &ap : pl.ap) ap.family = TAD_FAMILY_WORKED;
        pl.ws_bytes = worked_workspace_bytes(I, J, K);
        return true;
    }
    if (K % 32 == 0) {
        // long summed index: the contraction over k (and the collapsed j / i contractions of the gradients)
        // are dense matrix products and run on the matrix cores
        pl.fwd_family = TAD_FAMILY_WORKED_MFMA;
        for (auto &ap : pl.ap) ap.family = TAD_FAMILY_WORKED_MFMA;
        pl.ws_bytes = mfma_workspace_bytes(I, J, K);
        return true;
    }
    return false;
}

static bool unary_body(int body) {
    return body == TAD_BODY_SQ || body == TAD_BODY_CUBE || body == TAD_BODY_SIN || body == TAD_BODY_EXP;
}

// the three one-argument patterns of the introduction: f_ij = phi(x_i), f_i = phi(x_ii), f_ij = phi(x_{i+j})
static bool match_patterns(tad_plan &pl) {
    const tad_expr &e = pl.expr;
    if (!unary_body(e.body) || pl.dtype != TAD_F32 || e.n_sum != 0 || !all_derived(pl)) return false;
    const tad_arg &x = pl.args[0];
    const ArgPlan &px = pl.ap[0];
    int fam = TAD_FAMILY_GENERIC;
    if (e.n_f == 2 && index_is(x, 2, {{1, 0}})) {
        // kernel coordinate = j over its whole range, i = y_0
        if (e.f_shape[1] % 4 != 0 || px.smith.R != 1 || px.K.cols != 1) return false;
        if (px.VR(0, 0) != 1 || px.VR(1, 0) != 0 || px.K(0, 0) != 0 || px.K(1, 0) * px.K(1, 0) != 1) return false;
        if (!y_is_beta(px.dev) || !flatten_feas(px.dev, pl.fast.feas)) return false;
        fam = TAD_FAMILY_ROW_REDUCE;
    } else if (e.n_f == 1 && index_is(x, 1, {{1}, {1}})) {
        if (x.shape[1] % 4 != 0 || px.smith.R != 1 || px.K.cols != 0 || px.VR(0, 0) != 1) return false;
        // transformed index y = first gradient index; one cokernel row +-(1, -1)
        const GatherPlan &g = px.dev;
        if (g.nC != 1 || g.C[0][0] + g.C[0][1] != 0 || g.C[0][0] * g.C[0][0] != 1) return false;
        if (g.diag[0] != 1 || g.U[0][0] != 1 || g.U[0][1] != 0 || !flatten_feas(g, pl.fast.feas)) return false;
        pl.fast.c_ld = x.shape[1];
        fam = TAD_FAMILY_DIAGONAL;
    } else if (e.n_f == 2 && index_is(x, 2, {{1, 1}})) {
        if (e.f_shape[1] % 4 != 0 || px.smith.R != 1 || px.K.cols != 1) return false;
        if (px.K(0, 0) * px.K(0, 0) != 1 || px.K(1, 0) * px.K(1, 0) != 1) return false;
        if (!y_is_beta(px.dev) || !flatten_feas(px.dev, pl.fast.feas) || !flatten_level(px.dev, 0, pl.fast.flat[0]))
            return false;
        pl.fast.dd_iy = (int)px.VR(0, 0); pl.fast.dd_iz = (int)px.K(0, 0);
        pl.fast.jy = (int)px.VR(1, 0); pl.fast.jz = (int)px.K(1, 0);
        pl.ws_bytes = antidiag_workspace_bytes(e.f_shape[0], e.f_shape[1]);
        fam = TAD_FAMILY_ANTIDIAGONAL;
    } else {
        return false;
    }
    pl.fast.I = e.f_shape[0];
    pl.fast.J = e.n_f == 2 ? e.f_shape[1] : 1;
    pl.fwd_family = fam;
    pl.ap[0].family = fam;
    return true;
}

// f_nij = tanh(sum_{u,v} x_{n, s i + u, s j + v} w_uv), extended index (n, i, j, u, v)
static bool match_strided(tad_plan &pl) {
    const tad_expr &e = pl.expr;
    if (e.body != TAD_BODY_TANH_DOT || pl.dtype != TAD_F32 || e.n_f != 3 || e.n_sum != 2) return false;
    if (e.sum_lo[0] != 0 || e.sum_lo[1] != 0 || !all_derived(pl)) return false;
    const tad_arg &x = pl.args[0], &w = pl.args[1];
    if (x.rank != 3 || w.rank != 2) return false;
    const int64_t s = x.index[1][1];
    if (s < 1) return false;
    if (!index_is(x, 5, {{1, 0, 0, 0, 0}, {0, s, 0, 1, 0}, {0, 0, s, 0, 1}})) return false;
    if (!index_is(w, 5, {{0, 0, 0, 1, 0}, {0, 0, 0, 0, 1}})) return false;
    const int64_t U = e.sum_hi[0] + 1, V = e.sum_hi[1] + 1;
    if (w.shape[0] != U || w.shape[1] != V || U * V > 49) return false;
    // x: two kernel coordinates with plan-driven ranges; w: the three function indices collapse completely
    const ArgPlan &px = pl.ap[0], &pw = pl.ap[1];
    if (px.K.cols != 2 || pw.K.cols != 3 || px.smith.R != 3) return false;
    // x: y = beta, and both ranges in the loop-free form (neither depends on the other kernel coordinate)
    if (!y_is_beta(px.dev) || !flatten_feas(px.dev, pl.fast.feas)) return false;
    if (!flatten_level(px.dev, 0, pl.fast.flat[0]) || !flatten_level(px.dev, 1, pl.fast.flat[1])) return false;
    pl.fast.N = e.f_shape[0]; pl.fast.I = e.f_shape[1]; pl.fast.J = e.f_shape[2];
    pl.fast.U = U; pl.fast.V = V; pl.fast.stride = s;
    pl.fast.P = x.shape[1]; pl.fast.Q = x.shape[2];
    pl.fwd_family = TAD_FAMILY_STRIDED;
    pl.ap[0].family = pl.ap[1].family = TAD_FAMILY_STRIDED;
    pl.ws_bytes = strided_workspace_bytes(e.f_shape[0], e.f_shape[1], e.f_shape[2], U, V, s, x.shape[1], x.shape[2]);
    return true;
}

// f_ij = sum_k P(i, k) Q(k, j): both operands are matrices indexed by one function index and the summation index,
// their axes in either order, shapes exactly the index ranges.  Extended index (i, j, k).
// the body is the product of its two operands, summed: built in, or a program that says the same
static bool is_product_body(const tad_plan &pl) {
    if (pl.expr.body == TAD_BODY_MUL) return true;
    if (pl.expr.body != TAD_BODY_PROGRAM || pl.prog.n_operands != 2) return false;
    const DevProg &in = pl.prog.inner, &out = pl.prog.outer;
    return out.n == 1 && out.op[0] == P_SUM && in.n == 3 && in.result == 2 && in.op[0] == P_ARG &&
           in.op[1] == P_ARG && in.a[0] + in.a[1] == 1 && in.op[2] == P_MUL && in.a[2] + in.b[2] == 1;
}

static bool match_contraction(tad_plan &pl) {
    const tad_expr &e = pl.expr;
    if (!is_product_body(pl) || pl.dtype != TAD_F32 || e.n_f != 2 || e.n_sum != 1 || e.sum_lo[0] != 0) return false;
    if (!all_derived(pl)) return false;
    const int64_t ext[3] = {e.f_shape[0], e.f_shape[1], e.sum_hi[0] + 1};
    for (int d = 0; d < 3; ++d)
        if (ext[d] % 4 != 0 || ext[d] > (1 << 20)) return false;   // 16-byte rows; int32 addressing inside the kernel
    // axis_dim[p][r]: which extended index axis r of operand p follows (rows of the index matrix are unit vectors)
    int axis_dim[2][2];
    for (int p = 0; p < 2; ++p) {
        const tad_arg &a = pl.args[p];
        if (a.rank != 2) return false;
        for (int r = 0; r < 2; ++r) {
            int dim = -1;
            for (int d = 0; d < 3; ++d) {
                if (a.index[r][d] == 1 && dim < 0) dim = d;
                else if (a.index[r][d] != 0) return false;
            }
            if (dim < 0 || a.shape[r] != ext[dim]) return false;
            axis_dim[p][r] = dim;
        }
        if (axis_dim[p][0] == axis_dim[p][1]) return false;
    }
    auto has = [&](int p, int dim) { return axis_dim[p][0] == dim || axis_dim[p][1] == dim; };
    int P = -1, Q = -1;
    if (has(0, 0) && has(0, 2) && has(1, 1) && has(1, 2)) { P = 0; Q = 1; }
    else if (has(1, 0) && has(1, 2) && has(0, 1) && has(0, 2)) { P = 1; Q = 0; }
    else return false;
    // the derived plans must say what the kernels assume: y = beta, one kernel coordinate, and its range is the
    // whole collapsed dimension whatever beta is
    for (int p = 0; p < 2; ++p) {
        const ArgPlan &ap = pl.ap[p];
        const int gone = p == P ? 1 : 0;   // function index missing from the operand
        if (ap.smith.R != 2 || ap.K.cols != 1 || !y_is_beta(ap.dev)) return false;
        // no feasibility row may fail anywhere inside the operand's shape (no element is masked out)
        for (int r = 0; r < ap.dev.nF; ++r) {
            int64_t worst = ap.dev.feas[r].k0;
            for (int c = 0; c < 2; ++c) worst += std::max<int64_t>(0, (int64_t)ap.dev.feas[r].ky[c] * (ap.dev.shape[c] - 1));
            if (worst > 0) return false;
        }
        for (int d = 0; d < 3; ++d)
            if (ap.K(d, 0) * ap.K(d, 0) != (d == gone ? 1 : 0)) return false;
        FlatLevel fl;
        if (!flatten_level(ap.dev, 0, fl)) return false;
        for (int r = 0; r < kFlatRows; ++r)
            for (int c = 0; c < kFlatY; ++c)
                if (fl.lky[r][c] != 0 || fl.hky[r][c] != 0) return false;
        const int32_t y0[3] = {0, 0, 0};
        int32_t lo, hi;
        flat_bounds(fl, y0, lo, hi);
        if ((int64_t)hi - lo + 1 != ext[gone]) return false;
    }
    const int I = (int)ext[0], J = (int)ext[1], Kc = (int)ext[2];
    const bool p_ik = axis_dim[P][0] == 0;   // P stored [i][k]
    const bool q_kj = axis_dim[Q][0] == 2;   // Q stored [k][j]
    const int ldp = (int)pl.args[P].shape[1], ldq = (int)pl.args[Q].shape[1];
    GemmDesc *g = pl.fast.gemm;
    // f[i][j] = sum_k P(i,k) Q(k,j)
    g[0] = GemmDesc{I, J, Kc, P, Q, -1, ldp, ldq, !p_ik, !q_kj};
    // gradient of P in its own memory order
    if (p_ik) g[1] = GemmDesc{I, Kc, J, -1, Q, P, J, ldq, 0, q_kj};       // dP[i][k] = sum_j df[i][j] Q(k,j)
    else      g[1] = GemmDesc{Kc, I, J, Q, -1, P, ldq, J, !q_kj, 1};      // dP[k][i] = sum_j Q(k,j) df[i][j]
    // gradient of Q in its own memory order
    if (q_kj) g[2] = GemmDesc{Kc, J, I, P, -1, Q, ldp, J, p_ik, 0};       // dQ[k][j] = sum_i P(i,k) df[i][j]
    else      g[2] = GemmDesc{J, Kc, I, -1, P, Q, J, ldp, 1, !p_ik};      // dQ[j][k] = sum_i df[i][j] P(i,k)
    // A product with few output tiles and a long contraction index leaves most of the chip idle: cut the index
    // into pieces for separate workgroups (partial products in the workspace, added in a fixed order afterwards).
    size_t ws = 0;
    for (int q = 0; q < 3; ++q) {
        const long long tiles = (long long)((g[q].M + 127) / 128) * ((g[q].N + 127) / 128);
        int sp = 1;
        if (tiles < 256 && g[q].Kc >= 512) {
            sp = (int)std::min<long long>((512 + tiles - 1) / tiles, g[q].Kc / 256);
            sp = std::max(1, std::min(sp, 256));
        }
        g[q].splits = sp;
        if (sp > 1) ws = std::max(ws, align256((size_t)sp * g[q].M * g[q].N * sizeof(float)));
    }
    pl.ws_bytes = ws;
    pl.fwd_family = TAD_FAMILY_CONTRACTION;
    pl.ap[0].family = pl.ap[1].family = TAD_FAMILY_CONTRACTION;
    return true;
}

static void select_specialised(tad_plan &plan) {
    plan.fwd_family = TAD_FAMILY_GENERIC;
    for (auto &ap : plan.ap) ap.family = TAD_FAMILY_GENERIC;
    plan.ws_bytes = 0;
    if (plan.expr.body == TAD_BODY_PROGRAM) {
        // interpreter kernels; the backward pass keeps g = df * outer'(sum) for every function element
        plan.fwd_family = TAD_FAMILY_PROGRAM;
        for (auto &ap : plan.ap) ap.family = TAD_FAMILY_PROGRAM;
        // ... and, if the outer function reads operands, the sums themselves for the terms df * d outer / d x
        plan.ws_bytes = align256((size_t)plan.f_count * (plan.dtype == TAD_F64 ? 8 : 4)) * (plan.prog.outer_mask ? 2 : 1);
        // a plain product of two matrices (the form the derived expressions of a matrix product have) still
        // belongs on the matrix cores
        if (!(plan.flags & TAD_PLAN_GENERIC_ONLY) && !plan.has_alias && plan.expr.n_constraints == 0 &&
            match_contraction(plan)) {
            // the matcher has set the family and the workspace of the products
        }
        return;
    }
    if ((plan.flags & TAD_PLAN_GENERIC_ONLY) || plan.has_alias || plan.expr.n_constraints > 0) return;
    if (match_worked(plan)) return;
    if (match_patterns(plan)) return;
    if (match_strided(plan)) return;
    if (match_contraction(plan)) return;
}

void select_families(tad_plan &plan) {
    select_specialised(plan);
    // the fallback kernels share the elements of a gradient with few elements and long sums among several blocks:
    // room for their partial sums behind whatever the family keeps in the workspace
    bool fallback = true;
    for (const auto &ap : plan.ap) fallback = fallback && (ap.family == TAD_FAMILY_GENERIC || ap.family == TAD_FAMILY_PROGRAM);
    plan.split_ws_offset = plan.ws_bytes;
    if (!fallback) return;
    // ... and those of a forward sum with few function indices
    size_t most = cooperative_splits(plan.f_count, plan.terms_total) > 1
                      ? align256((size_t)plan.f_count * (size_t)cooperative_splits(plan.f_count, plan.terms_total) * 8)
                      : 0;
    for (size_t q = 0; q < plan.args.size(); ++q) {
        if (!plan.ap[q].derived) continue;   // no gradient planned for this operand
        const long long n = gather_launch_count(plan.ap[q].dev, plan.arg_count[(size_t)plan.root[q]]);
        most = std::max(most, split_workspace_bytes(n, gather_shape(plan.ap[q].dev, n, plan.terms_total).splits));
        if (plan.expr.body == TAD_BODY_PROGRAM && ((plan.prog.outer_mask >> q) & 1u)) {
            const long long no = gather_launch_count(plan.ap_outer[q].dev, plan.arg_count[(size_t)plan.root[q]]);
            most = std::max(most, split_workspace_bytes(no, cooperative_splits(no, (double)plan.f_count)));
        }
    }
    plan.ws_bytes += most;
}

}  // namespace tad
