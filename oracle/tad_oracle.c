/*
 * CPU oracle (TEST INFRASTRUCTURE ONLY -- never part of the product path).
 *
 * A plain, slow, fp64 evaluation of an element-wise defined tensor and of its
 * gradients, written straight from the definitions in the paper:
 *
 *   forward   Sec. 5.1 (definition of f_alpha through index maps A^p) and
 *             Sec. 5.2 (a summation inside f: the summation index is appended
 *             to alpha, giving the sum-extended index [alpha k]).
 *   backward  the "elementary approach" of Sec. 5.1: visit every function
 *             index (and, per Sec. 5.2, every summation index) and add
 *             df_alpha * d fhat / d x^p  into  dx^p at position Ahat^p [alpha k].
 *             This is the chain rule itself; it uses no index inversion, no
 *             Smith normal form and no Fourier-Motzkin elimination.
 *   gamma     the set  Gamma-hat(beta)  of Sec. 5.2 by exhaustive scan of the
 *             index box (used to check index plans).
 *
 * Indices are zero based (Sec. 6).  Tensors are dense row-major doubles.
 * Nothing here is shared with the GPU library: no headers, no tables.
 *
 * Scalar bodies  f = outer( sum_k inner(values) ):
 *   "sq"       inner = x            outer = s^2
 *   "cube"     inner = x            outer = s^3
 *   "sin"      inner = x            outer = sin s
 *   "exp"      inner = x            outer = exp s
 *   "mul"      inner = x*y          outer = s
 *   "worked"   inner = (a+b)^2 c + d^3   outer = exp(-s)      (Sec. 1, Sec. 6)
 *   "tanh_dot" inner = x*w          outer = tanh s
 *   "program"  inner and outer given as postfix programs over the operand values / the sum; their
 *              derivatives are taken by forward-mode differentiation with dual numbers (value and
 *              derivative carried together through every operation), the textbook rules of Sec. 2's
 *              elementary functions -- deliberately not the reverse accumulation the GPU library uses.
 *              The outer program may also read operands whose index does not depend on the summation
 *              indices, at the function index (Sec. 5.2, the sum-liberated function
 *              fhat = fbar(s(...), x^1_{A^1 alpha}, ...)): such an operand receives, per function index,
 *              the extra gradient term df_alpha * d fbar / d x.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_EXT 8   /* function indices + summation indices */
#define ORC_MAX_RANK 4
#define ORC_MAX_ARGS 6
#define ORC_MAX_COND 8

typedef struct {
    int rank;
    int64_t shape[ORC_MAX_RANK];
    int64_t A[ORC_MAX_RANK][ORC_MAX_EXT]; /* index matrix, columns: function then summation indices */
} orc_arg;

#define ORC_MAX_PROGRAM 64
/* postfix operation codes of a program body */
enum { O_CONST, O_ARG, O_SUM, O_ADD, O_SUB, O_MUL, O_DIV, O_NEG, O_EXP, O_LOG, O_SIN, O_COS, O_TANH, O_SQRT, O_POWI,
       O_STORE, /* copy the top of the stack into temporary iarg (the stack is unchanged) */
       O_LOAD   /* push temporary iarg */ };
#define ORC_MAX_TEMPS 16
typedef struct {
    int op;        /* O_* */
    int iarg;      /* operand index (O_ARG) or integer exponent (O_POWI) */
    double value;  /* O_CONST */
} orc_op;

typedef struct {
    char body[16];
    int n_f;                       /* number of function indices */
    int64_t f_shape[ORC_MAX_EXT];
    int n_sum;                     /* number of summation indices */
    int64_t sum_lo[ORC_MAX_EXT], sum_hi[ORC_MAX_EXT]; /* inclusive limits */
    int n_args;
    orc_arg args[ORC_MAX_ARGS];
    int n_inner, n_outer;          /* body "program" only */
    orc_op inner[ORC_MAX_PROGRAM], outer[ORC_MAX_PROGRAM];
    /* summation ranges that depend on other indices (Sec. 5.2): the term at the extended index x = [alpha k]
       belongs to the sum iff  cond[j][0..n_ext) . x + cond[j][n_ext] >= 0  for every j < n_cond */
    int n_cond;
    int64_t cond[ORC_MAX_COND][ORC_MAX_EXT + 1];
} orc_expr;

enum { B_SQ, B_CUBE, B_SIN, B_EXP, B_MUL, B_WORKED, B_TANH_DOT, B_PROGRAM, B_UNKNOWN };

static int body_id(const char *s) {
    if (!strcmp(s, "sq")) return B_SQ;
    if (!strcmp(s, "cube")) return B_CUBE;
    if (!strcmp(s, "sin")) return B_SIN;
    if (!strcmp(s, "exp")) return B_EXP;
    if (!strcmp(s, "mul")) return B_MUL;
    if (!strcmp(s, "worked")) return B_WORKED;
    if (!strcmp(s, "tanh_dot")) return B_TANH_DOT;
    if (!strcmp(s, "program")) return B_PROGRAM;
    return B_UNKNOWN;
}

static int body_nargs(int b) {
    switch (b) {
    case B_SQ: case B_CUBE: case B_SIN: case B_EXP: return 1;
    case B_MUL: case B_TANH_DOT: return 2;
    case B_WORKED: return 4;
    default: return -1;
    }
}

/* A value together with its derivative with respect to one chosen input. */
typedef struct { double v, d; } dual;

/*
 * Run a postfix program on dual numbers.  `args` are the operand values, `sum` the summed inner value (outer
 * program).  One input has derivative one -- operand `seed_arg` (none if negative), or the sum if `seed_sum`
 * is set --, every other input and every constant derivative zero.  A malformed program yields NaN.
 */
static dual run_program(const orc_op *ops, int n, const double *args, double sum, int seed_arg, int seed_sum) {
    dual st[ORC_MAX_PROGRAM + 1], tmp[ORC_MAX_TEMPS];
    int top = 0, have[ORC_MAX_TEMPS] = {0};
    const dual bad = {NAN, NAN};
    for (int i = 0; i < n; ++i) {
        const orc_op *o = &ops[i];
        dual r;
        if (o->op == O_CONST) { r.v = o->value; r.d = 0.0; }
        else if (o->op == O_ARG) { r.v = args[o->iarg]; r.d = (o->iarg == seed_arg) ? 1.0 : 0.0; }
        else if (o->op == O_SUM) { r.v = sum; r.d = seed_sum ? 1.0 : 0.0; }
        else if (o->op == O_STORE) {
            if (top < 1 || o->iarg < 0 || o->iarg >= ORC_MAX_TEMPS) return bad;
            tmp[o->iarg] = st[top - 1];
            have[o->iarg] = 1;
            continue;
        } else if (o->op == O_LOAD) {
            if (o->iarg < 0 || o->iarg >= ORC_MAX_TEMPS || !have[o->iarg]) return bad;
            r = tmp[o->iarg];
        }
        else if (o->op >= O_ADD && o->op <= O_DIV) {
            if (top < 2) return bad;
            dual y = st[--top], x = st[--top];
            if (o->op == O_ADD) { r.v = x.v + y.v; r.d = x.d + y.d; }
            else if (o->op == O_SUB) { r.v = x.v - y.v; r.d = x.d - y.d; }
            else if (o->op == O_MUL) { r.v = x.v * y.v; r.d = x.d * y.v + x.v * y.d; }
            else { r.v = x.v / y.v; r.d = (x.d - r.v * y.d) / y.v; }
        } else {
            if (top < 1) return bad;
            dual x = st[--top];
            switch (o->op) {
            case O_NEG: r.v = -x.v; r.d = -x.d; break;
            case O_EXP: r.v = exp(x.v); r.d = x.d * r.v; break;
            case O_LOG: r.v = log(x.v); r.d = x.d / x.v; break;
            case O_SIN: r.v = sin(x.v); r.d = x.d * cos(x.v); break;
            case O_COS: r.v = cos(x.v); r.d = -x.d * sin(x.v); break;
            case O_TANH: r.v = tanh(x.v); r.d = x.d * (1.0 - r.v * r.v); break;
            case O_SQRT: r.v = sqrt(x.v); r.d = x.d / (2.0 * r.v); break;
            case O_POWI: r.v = pow(x.v, (double)o->iarg); r.d = x.d * (double)o->iarg * pow(x.v, (double)(o->iarg - 1)); break;
            default: return bad;
            }
        }
        st[top++] = r;
    }
    return top == 1 ? st[0] : bad;
}

/* summand s(v) of the inner sum */
static double inner(const orc_expr *e, int b, const double *v) {
    if (b == B_PROGRAM) return run_program(e->inner, e->n_inner, v, 0.0, -1, 0).v;
    switch (b) {
    case B_MUL: case B_TANH_DOT: return v[0] * v[1];
    case B_WORKED: { double t = v[0] + v[1]; return t * t * v[2] + v[3] * v[3] * v[3]; }
    default: return v[0];
    }
}

/* d s / d v[p] */
static double dinner(const orc_expr *e, int b, int p, const double *v) {
    if (b == B_PROGRAM) return run_program(e->inner, e->n_inner, v, 0.0, p, 0).d;
    switch (b) {
    case B_MUL: case B_TANH_DOT: return p == 0 ? v[1] : v[0];
    case B_WORKED:
        if (p == 0 || p == 1) return 2.0 * (v[0] + v[1]) * v[2];
        if (p == 2) { double t = v[0] + v[1]; return t * t; }
        return 3.0 * v[3] * v[3];
    default: return 1.0;
    }
}

/* fbar(s, operand values at the function index); v is only read by programs */
static double outer(const orc_expr *e, int b, double s, const double *v) {
    if (b == B_PROGRAM) return run_program(e->outer, e->n_outer, v, s, -1, 0).v;
    switch (b) {
    case B_SQ: return s * s;
    case B_CUBE: return s * s * s;
    case B_SIN: return sin(s);
    case B_EXP: return exp(s);
    case B_MUL: return s;
    case B_WORKED: return exp(-s);
    case B_TANH_DOT: return tanh(s);
    default: return 0.0;
    }
}

/* d outer / d operand p (programs only; a built-in outer function takes no operands) */
static double douter_arg(const orc_expr *e, int b, double s, const double *v, int p) {
    if (b == B_PROGRAM) return run_program(e->outer, e->n_outer, v, s, p, 0).d;
    return 0.0;
}

/* d outer / d s */
static double douter(const orc_expr *e, int b, double s, const double *v) {
    if (b == B_PROGRAM) return run_program(e->outer, e->n_outer, v, s, -1, 1).d;
    switch (b) {
    case B_SQ: return 2.0 * s;
    case B_CUBE: return 3.0 * s * s;
    case B_SIN: return cos(s);
    case B_EXP: return exp(s);
    case B_MUL: return 1.0;
    case B_WORKED: return -exp(-s);
    case B_TANH_DOT: { double t = tanh(s); return 1.0 - t * t; }
    default: return 0.0;
    }
}

/* flat row-major position of argument p at extended index ext; -1 if outside its shape */
static int64_t arg_pos(const orc_arg *a, int n_ext, const int64_t *ext) {
    int64_t pos = 0;
    for (int r = 0; r < a->rank; ++r) {
        int64_t idx = 0;
        for (int d = 0; d < n_ext; ++d) idx += a->A[r][d] * ext[d];
        if (idx < 0 || idx >= a->shape[r]) return -1;
        pos = pos * a->shape[r] + idx;
    }
    return pos;
}

static int check_expr(const orc_expr *e, int *b) {
    *b = body_id(e->body);
    if (*b == B_UNKNOWN) return -1;
    if (*b == B_PROGRAM) {
        if (e->n_args < 1 || e->n_args > ORC_MAX_ARGS) return -2;
        if (e->n_inner < 1 || e->n_inner > ORC_MAX_PROGRAM || e->n_outer < 1 || e->n_outer > ORC_MAX_PROGRAM) return -5;
        for (int i = 0; i < e->n_inner; ++i)
            if (e->inner[i].op == O_SUM || (e->inner[i].op == O_ARG && (e->inner[i].iarg < 0 || e->inner[i].iarg >= e->n_args)))
                return -5;
        /* the outer function may read an operand only if its index ignores the summation indices */
        for (int i = 0; i < e->n_outer; ++i)
            if (e->outer[i].op == O_ARG) {
                int p = e->outer[i].iarg;
                if (p < 0 || p >= e->n_args) return -5;
                for (int r = 0; r < e->args[p].rank && r < ORC_MAX_RANK; ++r)
                    for (int q = 0; q < e->n_sum; ++q)
                        if (e->args[p].A[r][e->n_f + q] != 0) return -5;
            }
    } else if (e->n_args != body_nargs(*b)) return -2;
    if (e->n_f < 0 || e->n_sum < 0 || e->n_f + e->n_sum > ORC_MAX_EXT) return -3;
    if (e->n_cond < 0 || e->n_cond > ORC_MAX_COND) return -6;
    for (int p = 0; p < e->n_args; ++p)
        if (e->args[p].rank < 1 || e->args[p].rank > ORC_MAX_RANK) return -4;
    return 0;
}

/* does the extended index belong to the sum? */
static int in_range(const orc_expr *e, const int64_t *ext) {
    int n_ext = e->n_f + e->n_sum;
    for (int j = 0; j < e->n_cond; ++j) {
        int64_t v = e->cond[j][n_ext];
        for (int d = 0; d < n_ext; ++d) v += e->cond[j][d] * ext[d];
        if (v < 0) return 0;
    }
    return 1;
}

static int64_t f_count(const orc_expr *e) {
    int64_t n = 1;
    for (int d = 0; d < e->n_f; ++d) n *= e->f_shape[d];
    return n;
}

static void unflatten_f(const orc_expr *e, int64_t lin, int64_t *ext) {
    for (int d = e->n_f - 1; d >= 0; --d) { ext[d] = lin % e->f_shape[d]; lin /= e->f_shape[d]; }
}

/* advance the summation part of ext (odometer, last index fastest); returns 0 when exhausted */
static int next_sum(const orc_expr *e, int64_t *ext) {
    for (int s = e->n_sum - 1; s >= 0; --s) {
        int d = e->n_f + s;
        if (ext[d] < e->sum_hi[s]) { ext[d]++; return 1; }
        ext[d] = e->sum_lo[s];
    }
    return 0;
}

static int sums_empty(const orc_expr *e) {
    for (int s = 0; s < e->n_sum; ++s) if (e->sum_lo[s] > e->sum_hi[s]) return 1;
    return 0;
}

/* s_alpha = sum over the summation box of inner(values), ascending index order */
static int eval_s(const orc_expr *e, int b, const double *const *args, int64_t *ext, double *s_out) {
    int n_ext = e->n_f + e->n_sum;
    double s = 0.0, v[ORC_MAX_ARGS];
    if (!sums_empty(e)) {
        for (int q = 0; q < e->n_sum; ++q) ext[e->n_f + q] = e->sum_lo[q];
        do {
            if (!in_range(e, ext)) continue;
            for (int p = 0; p < e->n_args; ++p) {
                int64_t pos = arg_pos(&e->args[p], n_ext, ext);
                if (pos < 0) return -10;
                v[p] = args[p][pos];
            }
            s += inner(e, b, v);
        } while (next_sum(e, ext));
    }
    *s_out = s;
    return 0;
}

/* is operand p read by the outer program? */
static int in_outer(const orc_expr *e, int b, int p) {
    if (b != B_PROGRAM) return 0;
    for (int i = 0; i < e->n_outer; ++i)
        if (e->outer[i].op == O_ARG && e->outer[i].iarg == p) return 1;
    return 0;
}

/* values (and positions) of the operands the outer program reads, at the function index in ext */
static int outer_values(const orc_expr *e, int b, const double *const *args, int64_t *ext, double *v, int64_t *pos) {
    int n_ext = e->n_f + e->n_sum;
    for (int q = 0; q < e->n_sum; ++q) ext[e->n_f + q] = e->sum_lo[q];   /* any value: those columns are zero */
    for (int p = 0; p < e->n_args; ++p) {
        v[p] = 0.0;
        pos[p] = -1;
        if (!in_outer(e, b, p)) continue;
        pos[p] = arg_pos(&e->args[p], n_ext, ext);
        if (pos[p] < 0) return -10;
        v[p] = args[p][pos[p]];
    }
    return 0;
}

/* Forward: f_alpha for every alpha (Sec. 5.1, 5.2). */
int orc_forward(const orc_expr *e, const double *const *args, double *f) {
    int b, rc = check_expr(e, &b);
    if (rc) return rc;
    int64_t nf = f_count(e);
    int err = 0;
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < nf; ++lin) {
        int64_t ext[ORC_MAX_EXT];
        double s, vo[ORC_MAX_ARGS];
        int64_t po[ORC_MAX_ARGS];
        unflatten_f(e, lin, ext);
        if (eval_s(e, b, args, ext, &s) || outer_values(e, b, args, ext, vo, po)) { err = -10; continue; }
        f[lin] = outer(e, b, s, vo);
    }
    return err;
}

/*
 * Backward by brute-force scatter (Sec. 5.1 "elementary approach", with the
 * sum-extended index set of Sec. 5.2):
 *   for every alpha, every k:   dx^p[ Ahat^p [alpha k] ] += df_alpha * outer'(s_alpha) * d inner / d x^p
 *   for every alpha, every operand the outer function reads:   dx^p[ A^p alpha ] += df_alpha * d outer / d x^p
 * dx[p] may be NULL (gradient not wanted).  dx[p] is overwritten.
 * With nthreads > 1 the function indices are split in contiguous chunks, every
 * thread scatters into private copies which are then added in thread order.
 */
int orc_backward(const orc_expr *e, const double *const *args, const double *df,
                 double *const *dx, int nthreads) {
    int b, rc = check_expr(e, &b);
    if (rc) return rc;
    int n_ext = e->n_f + e->n_sum;
    int64_t nf = f_count(e);
    int64_t asz[ORC_MAX_ARGS];
    for (int p = 0; p < e->n_args; ++p) {
        asz[p] = 1;
        for (int r = 0; r < e->args[p].rank; ++r) asz[p] *= e->args[p].shape[r];
        if (dx[p]) memset(dx[p], 0, (size_t)asz[p] * sizeof(double));
    }
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > nf) nthreads = nf > 0 ? (int)nf : 1;
    double **priv = (double **)calloc((size_t)nthreads * ORC_MAX_ARGS, sizeof(double *));
    if (!priv) return -20;
    int err = 0;
    for (int t = 0; t < nthreads; ++t)
        for (int p = 0; p < e->n_args; ++p) {
            if (!dx[p]) continue;
            if (t == 0) { priv[p] = dx[p]; continue; }
            priv[t * ORC_MAX_ARGS + p] = (double *)calloc((size_t)asz[p], sizeof(double));
            if (!priv[t * ORC_MAX_ARGS + p]) err = -20;
        }
    if (!err) {
#pragma omp parallel for schedule(static, 1) num_threads(nthreads)
        for (int t = 0; t < nthreads; ++t) {
            int64_t lo = nf * t / nthreads, hi = nf * (t + 1) / nthreads;
            double **my = priv + t * ORC_MAX_ARGS;
            int64_t ext[ORC_MAX_EXT];
            double v[ORC_MAX_ARGS], vo[ORC_MAX_ARGS];
            int64_t pos[ORC_MAX_ARGS], po[ORC_MAX_ARGS];
            for (int64_t lin = lo; lin < hi; ++lin) {
                double s;
                unflatten_f(e, lin, ext);
                if (eval_s(e, b, args, ext, &s) || outer_values(e, b, args, ext, vo, po)) { err = -10; break; }
                double w = df[lin] * douter(e, b, s, vo);
                for (int p = 0; p < e->n_args; ++p)
                    if (my[p] && po[p] >= 0) my[p][po[p]] += df[lin] * douter_arg(e, b, s, vo, p);
                if (sums_empty(e)) continue;
                for (int q = 0; q < e->n_sum; ++q) ext[e->n_f + q] = e->sum_lo[q];
                do {
                    if (!in_range(e, ext)) continue;
                    for (int p = 0; p < e->n_args; ++p) {
                        pos[p] = arg_pos(&e->args[p], n_ext, ext);
                        v[p] = args[p][pos[p]];
                    }
                    for (int p = 0; p < e->n_args; ++p)
                        if (my[p]) my[p][pos[p]] += w * dinner(e, b, p, v);
                } while (next_sum(e, ext));
            }
        }
        for (int t = 1; t < nthreads; ++t)
            for (int p = 0; p < e->n_args; ++p) {
                double *src = priv[t * ORC_MAX_ARGS + p];
                if (!src) continue;
                for (int64_t i = 0; i < asz[p]; ++i) dx[p][i] += src[i];
            }
    }
    for (int t = 1; t < nthreads; ++t)
        for (int p = 0; p < e->n_args; ++p) free(priv[t * ORC_MAX_ARGS + p]);
    free(priv);
    return err;
}

/* lexicographic scan of the whole extended index box; calls back with every point */
static int box_first(const orc_expr *e, int64_t *ext) {
    for (int d = 0; d < e->n_f; ++d) { if (e->f_shape[d] <= 0) return 0; ext[d] = 0; }
    for (int s = 0; s < e->n_sum; ++s) {
        if (e->sum_lo[s] > e->sum_hi[s]) return 0;
        ext[e->n_f + s] = e->sum_lo[s];
    }
    return 1;
}

static int box_next(const orc_expr *e, int64_t *ext) {
    for (int d = e->n_f + e->n_sum - 1; d >= 0; --d) {
        int64_t lo = d < e->n_f ? 0 : e->sum_lo[d - e->n_f];
        int64_t hi = d < e->n_f ? e->f_shape[d] - 1 : e->sum_hi[d - e->n_f];
        if (ext[d] < hi) { ext[d]++; return 1; }
        ext[d] = lo;
    }
    return 0;
}

/*
 * Gamma-hat(beta) of Sec. 5.2 for argument `arg`: every extended index in the
 * box whose image under Ahat equals beta, in lexicographic order.  Writes up to
 * `cap` points (n_ext values each) into out and the total count into *n.
 */
int orc_gamma(const orc_expr *e, int arg, const int64_t *beta, int64_t *out, int64_t cap, int64_t *n) {
    int b, rc = check_expr(e, &b);
    if (rc) return rc;
    if (arg < 0 || arg >= e->n_args) return -5;
    const orc_arg *a = &e->args[arg];
    int n_ext = e->n_f + e->n_sum;
    int64_t ext[ORC_MAX_EXT], cnt = 0;
    if (box_first(e, ext)) {
        do {
            int hit = in_range(e, ext);
            for (int r = 0; r < a->rank && hit; ++r) {
                int64_t idx = 0;
                for (int d = 0; d < n_ext; ++d) idx += a->A[r][d] * ext[d];
                hit = idx == beta[r];
            }
            if (hit) {
                if (cnt < cap) memcpy(out + cnt * n_ext, ext, (size_t)n_ext * sizeof(int64_t));
                cnt++;
            }
        } while (box_next(e, ext));
    }
    *n = cnt;
    return 0;
}

/*
 * |Gamma-hat(beta)| for every beta of argument `arg` in one scan of the box:
 * counts[flat(beta)] = number of extended indices mapped onto beta.
 * counts has one int64 per element of the argument and is overwritten.
 */
int orc_gamma_counts(const orc_expr *e, int arg, int64_t *counts) {
    int b, rc = check_expr(e, &b);
    if (rc) return rc;
    if (arg < 0 || arg >= e->n_args) return -5;
    const orc_arg *a = &e->args[arg];
    int n_ext = e->n_f + e->n_sum;
    int64_t sz = 1;
    for (int r = 0; r < a->rank; ++r) sz *= a->shape[r];
    memset(counts, 0, (size_t)sz * sizeof(int64_t));
    int64_t ext[ORC_MAX_EXT];
    if (box_first(e, ext)) {
        do {
            if (!in_range(e, ext)) continue;
            int64_t pos = arg_pos(a, n_ext, ext);
            if (pos < 0) return -10;
            counts[pos]++;
        } while (box_next(e, ext));
    }
    return 0;
}

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int orc_sizeof_expr(void) { return (int)sizeof(orc_expr); }
