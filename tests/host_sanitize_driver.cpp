// Host-only driver for the address / undefined-behaviour sanitizer run of the index planner
// (tests/test_host_sanitizers.py builds it together with plan.cpp, derived.cpp and families.cpp; no GPU code).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/tad.h"
#include "../paper_1711_01348_amd/csrc/plan_dev.h"

static int derive_worked(int64_t I, int64_t J, int64_t K, tad_dtype dt, uint32_t flags) {
    tad_expr e;
    std::memset(&e, 0, sizeof e);
    e.body = TAD_BODY_WORKED; e.n_f = 2; e.f_shape[0] = I; e.f_shape[1] = J; e.n_sum = 1; e.sum_lo[0] = 0; e.sum_hi[0] = K - 1;
    tad_arg a[4];
    std::memset(a, 0, sizeof a);
    const int64_t idx[4][2][3] = {{{1, 0, 0}, {0, 0, 1}}, {{0, 1, 0}, {0, 0, 1}}, {{1, 0, 0}, {1, 0, 0}}, {{1, 0, 1}, {0, 0, 0}}};
    const int64_t shp[4][2] = {{I, K}, {J, K}, {I, I}, {I + K - 1, 0}};
    for (int p = 0; p < 4; ++p) {
        a[p].rank = p == 3 ? 1 : 2; a[p].needs_grad = 1;
        for (int r = 0; r < a[p].rank; ++r) {
            a[p].shape[r] = shp[p][r];
            for (int d = 0; d < 3; ++d) a[p].index[r][d] = idx[p][r][d];
        }
    }
    tad_plan *pl = nullptr;
    int rc = tad_plan_derive(&e, a, 4, dt, flags, &pl);
    if (rc) return rc;
    // walk the plan: query, rows, enumeration of every gradient element of d and a few of c
    for (int p = 0; p < 4; ++p) {
        tad_plan_info info;
        if (tad_plan_query(pl, p, 0, &info)) return -100;
        int64_t scale, cb[2 * TAD_MAX_EXT], cz[TAD_MAX_KERNEL];
        for (int lvl = 0; lvl < info.kernel_dim; ++lvl)
            for (int r = 0; r < info.n_lower[lvl]; ++r)
                if (tad_plan_bound_row(pl, p, TAD_ROWS_LOWER, lvl, r, &scale, cb, cz, nullptr)) return -101;
    }
    std::vector<int64_t> buf((size_t)J * K * 3 + 3);
    for (int64_t m = 0; m < I + K - 1; ++m) {
        size_t n = 0;
        if (tad_plan_enumerate(pl, 3, 0, &m, buf.data(), (size_t)J * K, &n)) return -102;
    }
    const int64_t beta[2] = {I - 1, I - 1};
    size_t n = 0;
    if (tad_plan_enumerate(pl, 2, 0, beta, buf.data(), (size_t)J * K, &n) || n != (size_t)(J * K)) return -103;
    std::vector<int64_t> counts((size_t)I * I);
    if (tad_plan_count_all(pl, 2, counts.data())) return -104;
    (void)tad_plan_workspace_bytes(pl);
    tad_plan_free(pl);
    return 0;
}

int main() {
    if (derive_worked(8, 6, 5, TAD_F64, 0)) return 1;
    if (derive_worked(333, 1300, 5, TAD_F32, 0)) return 2;
    if (derive_worked(64, 128, 256, TAD_F32, 0)) return 3;
    if (derive_worked(40, 44, 7, TAD_F32, TAD_PLAN_GENERIC_ONLY)) return 4;
    // integer machinery on awkward inputs
    unsigned seed = 12345;
    auto rnd = [&]() { seed = seed * 1664525u + 1013904223u; return (int)((seed >> 16) % 9) - 4; };
    for (int t = 0; t < 400; ++t) {
        const int n = 1 + (t % 3), m = 1 + (t % 4);
        int64_t A[12], lo[4], hi[4], beta[3];
        bool nz = false;
        for (int i = 0; i < n * m; ++i) { A[i] = rnd(); nz |= A[i] != 0; }
        if (!nz) continue;
        for (int d = 0; d < m; ++d) { lo[d] = rnd() / 2; hi[d] = lo[d] + (rnd() + 4) / 2; }
        for (int r = 0; r < n; ++r) beta[r] = rnd();
        int64_t S[12], U[9], V[16], out[4 * 4096];
        int R = 0;
        if (tad_smith_normal_form(A, n, m, S, U, V, &R)) return 5;
        size_t cnt = 0;
        const int rc = tad_lattice_enumerate(A, n, m, lo, hi, beta, out, 4096, &cnt);
        if (rc != 0 && rc != TAD_EUNSUPPORTED) return 6;
    }
    // overflow paths must report, not trap
    const int64_t big = (int64_t)1 << 62;
    int64_t Ab[4] = {big, big - 1, big - 3, big - 7}, S[4], U[4], V[4];
    int R = 0;
    if (tad_smith_normal_form(Ab, 2, 2, S, U, V, &R) != TAD_EOVERFLOW) return 7;
    int64_t g, x, y;
    if (tad_extended_gcd(INT64_MIN, 3, &g, &x, &y) != TAD_EOVERFLOW) return 8;
    // scalar bodies as programs: parsing, reverse accumulation, lowering, host evaluation
    {
        tad_expr e;
        std::memset(&e, 0, sizeof e);
        e.body = TAD_BODY_PROGRAM; e.n_f = 1; e.f_shape[0] = 5; e.n_operands = 2;
        const tad_op inner[] = {{TAD_OP_ARG, 0, 0}, {TAD_OP_ARG, 1, 0}, {TAD_OP_ARG, 0, 0}, {TAD_OP_SUB, 0, 0}, {TAD_OP_DIV, 0, 0},
                                {TAD_OP_ARG, 1, 0}, {TAD_OP_SQRT, 0, 0}, {TAD_OP_ARG, 0, 0}, {TAD_OP_POWI, 5, 0}, {TAD_OP_MUL, 0, 0},
                                {TAD_OP_SUB, 0, 0}, {TAD_OP_TANH, 0, 0}, {TAD_OP_CONST, 0, 1.5}, {TAD_OP_MUL, 0, 0}};
        const tad_op outer[] = {{TAD_OP_SUM, 0, 0}, {TAD_OP_COS, 0, 0}, {TAD_OP_NEG, 0, 0}, {TAD_OP_EXP, 0, 0}, {TAD_OP_LOG, 0, 0}};
        e.n_inner = (int)(sizeof inner / sizeof inner[0]); e.n_outer = (int)(sizeof outer / sizeof outer[0]);
        std::memcpy(e.inner, inner, sizeof inner);
        std::memcpy(e.outer, outer, sizeof outer);
        tad_arg a[2];
        std::memset(a, 0, sizeof a);
        for (int p = 0; p < 2; ++p) { a[p].rank = 1; a[p].shape[0] = 5; a[p].index[0][0] = 1; a[p].needs_grad = 1; }
        tad_plan *pl = nullptr;
        if (tad_plan_derive(&e, a, 2, TAD_F64, 0, &pl)) return 13;
        const double v[2] = {0.4, 1.3};
        double o = 0;
        for (int which = -3; which < 2; ++which)
            if (tad_plan_program_eval(pl, which, v, 0.7, &o) || o != o) return 14;
        if (tad_plan_program_eval(pl, 2, v, 0.7, &o) != TAD_EINVAL) return 15;
        tad_plan_free(pl);
        // malformed programs are refused
        e.n_inner = 2;   // ARG ARG: two values left
        if (tad_plan_derive(&e, a, 2, TAD_F64, 0, &pl) != TAD_EINVAL) return 16;
        e.n_inner = TAD_MAX_PROGRAM + 1;
        if (tad_plan_derive(&e, a, 2, TAD_F64, 0, &pl) != TAD_EINVAL) return 17;
    }
    // summation range that depends on another index: f_i = sum_{k <= i} x_{i-k} w_k
    {
        tad_expr e;
        std::memset(&e, 0, sizeof e);
        e.body = TAD_BODY_MUL; e.n_f = 1; e.f_shape[0] = 9; e.n_sum = 1; e.sum_lo[0] = 0; e.sum_hi[0] = 3;
        e.n_constraints = 1; e.constraint[0][0] = 1; e.constraint[0][1] = -1; e.constraint[0][2] = 0;
        tad_arg a[2];
        std::memset(a, 0, sizeof a);
        a[0].rank = 1; a[0].shape[0] = 9; a[0].index[0][0] = 1; a[0].index[0][1] = -1; a[0].needs_grad = 1;
        a[1].rank = 1; a[1].shape[0] = 4; a[1].index[0][1] = 1; a[1].needs_grad = 1;
        tad_plan *pl = nullptr;
        if (tad_plan_derive(&e, a, 2, TAD_F64, 0, &pl)) return 18;
        int64_t total = 0, buf[64 * 2];
        for (int64_t m = 0; m < 9; ++m) {
            size_t n = 0;
            if (tad_plan_enumerate(pl, 0, 0, &m, buf, 64, &n)) return 19;
            total += (int64_t)n;
        }
        if (total != 4 + 4 + 4 + 4 + 4 + 4 + 3 + 2 + 1) return 20;   // pairs (i, k) with k <= min(i, 3), grouped by i - k
        // each gradient as an expression of its own, planned again, and the gradients of that once more
        for (int p = 0; p < 2; ++p) {
            tad_expr de;
            tad_arg da[TAD_MAX_ARGS];
            int src[TAD_MAX_ARGS], n = 0;
            if (tad_plan_derived_expr(pl, p, 0, 0, &de, da, src, &n) || n != 2 || src[0] != -1 || src[1] != 1 - p) return 22;
            if (tad_plan_derived_expr(pl, p, 1, 0, &de, da, src, &n) != TAD_EINVAL) return 23;
            if (tad_plan_derived_expr(pl, p, 0, 1, &de, da, src, &n) != TAD_EINVAL) return 28;   // no outer operand
            tad_plan *dp = nullptr;
            if (tad_plan_derive(&de, da, n, TAD_F64, 0, &dp)) return 24;
            for (int q = 0; q < n; ++q) {
                tad_expr de2;
                tad_arg da2[TAD_MAX_ARGS];
                int n2 = 0;
                if (tad_plan_derived_expr(dp, q, 0, 0, &de2, da2, nullptr, &n2) || n2 != 2) return 25;
                tad_plan *dp2 = nullptr;
                if (tad_plan_derive(&de2, da2, n2, TAD_F64, 0, &dp2)) return 26;
                tad_plan_free(dp2);
            }
            tad_plan_free(dp);
        }
        if (tad_plan_derived_expr(pl, 0, 0, 0, nullptr, nullptr, nullptr, nullptr) != TAD_EINVAL) return 27;
        {
            tad_expr se;
            tad_arg sa[TAD_MAX_ARGS];
            int n = 0;
            if (tad_plan_seed_expr(pl, -1, &se, sa, &n) || n != 3) return 29;
            tad_plan *sp = nullptr;
            if (tad_plan_derive(&se, sa, n, TAD_F64, 0, &sp)) return 30;
            tad_plan_free(sp);
            if (tad_plan_seed_expr(pl, 0, &se, sa, &n) != TAD_EINVAL) return 31;
        }
        tad_plan_free(pl);
        e.n_constraints = 0;   // without the condition the index i - k can be negative
        if (tad_plan_derive(&e, a, 2, TAD_F64, 0, &pl) != TAD_ESHAPE) return 21;
    }
    // the loop-free floor division is exact on its whole domain (|a| < 2^23, 0 < s < 2^23)
    {
        const int32_t lim = (1 << 23) - 1;
        unsigned st = 99;
        auto next = [&]() { st = st * 1664525u + 1013904223u; return st; };
        auto exact = [](int64_t a, int64_t s) { int64_t q = a / s; if (a % s != 0 && a < 0) --q; return (int32_t)q; };
        for (int32_t s = 1; s <= 64; ++s) {
            const float rs = 1.f / (float)s;
            for (int32_t a = -lim; a <= lim; a += (s <= 8 ? 1 : 97)) {
                if (tad::floor_div_flat(a, s, rs) != exact(a, s)) return 9;
                if (tad::floor_div_float(a, s, rs) != exact(a, s)) return 13;   // also exact for the divisors 1 and 2
            }
            for (int32_t a : {-lim, -lim + 1, -s, -s - 1, -s + 1, -1, 0, 1, s - 1, s, s + 1, lim - 1, lim})
                if (tad::floor_div_flat(a, s, rs) != exact(a, s)) return 10;
        }
        for (int t = 0; t < 2000000; ++t) {
            const int32_t s = 1 + (int32_t)(next() % (unsigned)lim);
            const int32_t a = (int32_t)(next() % (2u * lim + 1)) - lim;
            if (tad::floor_div_flat(a, s, 1.f / (float)s) != exact(a, s)) return 11;
            // multiples of s and their neighbours are the hard cases
            const int32_t m = (int32_t)((int64_t)(a / s) * s);
            for (int32_t d = -1; d <= 1; ++d)
                if (m + d >= -lim && m + d <= lim && tad::floor_div_flat(m + d, s, 1.f / (float)s) != exact(m + d, s)) return 12;
        }
    }
    std::puts("sanitizer driver ok");
    return 0;
}
