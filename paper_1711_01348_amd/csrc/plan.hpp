// Host-side index plan: result of the element-wise derivation (Sec. 5.3) for
// every argument of one expression.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/tad.h"
#include "fm.hpp"
#include "plan_dev.h"
#include "program.hpp"
#include "snf.hpp"

namespace tad {

struct ArgPlan {
    bool derived = false;
    Smith smith;                 // S = U A V
    IMat UR, VR, K, C;           // first R rows of U, first R columns of V, kernel, cokernel
    IMat Vinv;                   // inverse of V: [y z] = Vinv [alpha k]
    std::vector<int64_t> diag;   // alpha_1..alpha_R
    FMResult fm;                 // rows over b(beta) in the paper's form
    GatherPlan dev;              // folded form used by kernels and by enumeration
    int family = TAD_FAMILY_GENERIC;
};

// One dense product C[m][n] = sum_k A(m, k) B(k, n) of the contraction family.  a_src / b_src: operand index,
// or -1 for df; out: operand index of the gradient written, or -1 for f.  at: A is stored [k][m]; bt: B is
// stored [n][k]; lda / ldb: row length of the stored matrix.
struct GemmDesc {
    int M = 0, N = 0, Kc = 0;
    int a_src = 0, b_src = 0, out = 0;
    int lda = 0, ldb = 0;
    int at = 0, bt = 0;
    int splits = 1;   // pieces of the contraction index computed by separate workgroups (few output tiles, long sum)
};

// Parameters of the specialised kernel families (filled by pattern recognition).
struct FastParams {
    int64_t I = 0, J = 0, K = 0;     // worked expression / 2-D patterns
    int64_t N = 0, U = 0, V = 0, stride = 0, P = 0, Q = 0;  // strided stencil
    int64_t c_ld = 0;                // row length of c (diagonal gather stride is c_ld + 1)
    // gradient of d: which kernel coordinate is the clipped window, and i = dd_iy * y_0 + dd_iz * z_window
    int dd_level = 0, dd_iy = 0, dd_iz = 0;
    int jy = 0, jz = 0;              // antidiagonal pattern: j = jy * y_0 + jz * z
    FlatLevel flat[2];               // loop-free range rows of the family's plan-driven coordinates
    FlatFeas feas;
    GemmDesc gemm[3];                // contraction family: forward, gradient of the i-operand, of the j-operand
};

}  // namespace tad

struct tad_plan {
    tad_expr expr;
    std::vector<tad_arg> args;
    tad_dtype dtype;
    uint32_t flags;
    int n_ext;
    int64_t lo[TAD_MAX_EXT], hi[TAD_MAX_EXT];  // inclusive box of the extended index
    int64_t f_count;
    double terms_total = 0;                    // extended indices in the box: f_count times the summation box
    std::vector<int64_t> arg_count;
    std::vector<int> root;                     // operand that holds the tensor of operand p (p itself unless alias)
    bool has_alias = false;
    tad::ForwardPlan fwd;
    std::vector<tad::ArgPlan> ap;
    // program bodies whose outer function reads operands: plan of such an operand over the function indices
    // alone (its index ignores the summation indices), for the gradient term df * d outer / d x
    std::vector<tad::ArgPlan> ap_outer;
    int fwd_family = TAD_FAMILY_GENERIC;
    tad::FastParams fast;
    tad::ProgramBody prog;                     // TAD_BODY_PROGRAM only
    std::vector<tad::TermList> term_list;      // one entry if the terms of every gradient element are listed (small expressions)
    size_t ws_bytes = 0;
    size_t split_ws_offset = 0;                // fallback kernels: where the partial sums of shared elements start
};

namespace tad {
// Loop-free copies of one level's range rows / of the feasibility rows; false if the plan does not fit
// (more rows than the fixed form holds, dependence on an outer kernel coordinate, more than kFlatY y's).
bool flatten_level(const GatherPlan &g, int level, FlatLevel &out);
bool flatten_feas(const GatherPlan &g, FlatFeas &out);
// true if the transformed index is the gradient index itself (U = 1, unit Smith diagonal, no cokernel)
bool y_is_beta(const GatherPlan &g);

// Derivation proper; throws tad::overflow_error on int64 overflow.
int derive_plan(const tad_expr *expr, const tad_arg *args, int n_args, tad_dtype dt, uint32_t flags,
                tad_plan **out);
int body_arg_count(int body);
// plan of occurrence `occ` of the tensor given as operand `arg`, and the operand slot of that occurrence
const ArgPlan *get_arg(const tad_plan *plan, int arg, int occ, int *slot_out = nullptr);
// Range of the linear form a . x over the rational relaxation of { lo <= x <= hi, extra conditions }; false if
// the set is empty.  The integer range is inside [tmin, tmax].
bool linear_form_range(const int64_t *a, int D, const int64_t *lo, const int64_t *hi, int E,
                       const int64_t (*cons_in)[TAD_MAX_EXT + 1], int64_t &tmin, int64_t &tmax);
// Pattern recognition of the specialised kernel families (device-independent; defined in families.cpp).
void select_families(tad_plan &plan);
}  // namespace tad
