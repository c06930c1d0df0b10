/*
 * tad.h -- C ABI of the tensor-algebra autodiff hot path (single GPU, gfx950).
 *
 * The library evaluates a tensor that is defined element-wise,
 *
 *     f_alpha = fbar( sum_{k in Psi} s( x^1_{A^1 [alpha k]}, ..., x^P_{A^P [alpha k]} ) ),
 *
 * (Sec. 5.1, and Sec. 5.2 for summations inside f), and the gradients
 * dx^p_beta = dl/dx^p_beta of a scalar loss l(f) for every argument, in the
 * gather form of Sec. 5.1 (final formula of that section):
 *
 *     dx^p_beta = delta(C beta) * sum_{z in Sigma(beta)} df_alpha * d fhat / d x^p  at  [alpha k] = I beta + K z,
 *
 * with I, K, C the pseudo-inverse, kernel and cokernel of the integer index
 * matrix A^p (Sec. 4.1, Smith normal form) and the nested ranges Sigma(beta)
 * obtained by Fourier-Motzkin elimination (Sec. 4.2).  One owner per gradient
 * element: no scatter, no atomics, bit-identical results from run to run.
 *
 * Conventions (all entry points):
 *   - indices are zero based (Sec. 6); summation limits are inclusive;
 *   - every tensor is dense, row-major (last index fastest), of the plan's dtype;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory of the current device, owned by the caller;
 *   - every function returns 0 on success or a negative tad_status; nothing
 *     throws, aborts or prints.
 */
#ifndef TAD_H
#define TAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TAD_MAX_EXT 6    /* function indices + summation indices */
#define TAD_MAX_RANK 4   /* rank of an argument tensor */
#define TAD_MAX_ARGS 6
#define TAD_MAX_KERNEL 4 /* dimension of the kernel of an index matrix */
#define TAD_MAX_CONSTRAINTS 8 /* extra linear conditions on the extended index */

typedef enum {
    TAD_OK = 0,
    TAD_EINVAL = -1,       /* NULL pointer, rank/size out of the supported limits, zero index matrix */
    TAD_ESHAPE = -2,       /* an index leaves its argument's shape; summation lo > hi; empty tensor */
    TAD_EINFEASIBLE = -3,  /* constraint system without any solution (Sec. 4.2, feasibility rows) */
    TAD_EOVERFLOW = -4,    /* integer overflow in Smith / Fourier-Motzkin, or index range beyond int32 */
    TAD_EUNSUPPORTED = -5, /* body / pattern without a kernel, plan beyond the fixed device limits */
    TAD_EDEVICE = -6,      /* kernel launch failed */
    TAD_ENOMEM = -7        /* host allocation failed, or workspace too small */
} tad_status;

typedef enum { TAD_F32 = 0, TAD_F64 = 1 } tad_dtype;

/*
 * Built-in scalar bodies  f = outer( sum_k inner(values) ).
 * Bodies SQ, CUBE and SIN take no summation index.
 */
typedef enum {
    TAD_BODY_SQ = 0,       /* x^2                                   (Sec. 1)            1 argument  */
    TAD_BODY_CUBE = 1,     /* x^3                                   (Sec. 5, f^3)       1 argument  */
    TAD_BODY_SIN = 2,      /* sin x                                 (Sec. 5, f^1)       1 argument  */
    TAD_BODY_EXP = 3,      /* exp(sum x)                            (Sec. 1, Sec. 5 f^5) 1 argument */
    TAD_BODY_MUL = 4,      /* sum x*y                               (Sec. 5, f^2, f^4)  2 arguments */
    TAD_BODY_WORKED = 5,   /* exp(-sum((a+b)^2 c + d^3))            (Sec. 1, Sec. 6)    4 arguments a,b,c,d */
    TAD_BODY_TANH_DOT = 6, /* tanh(sum x*w)                                             2 arguments x,w */
    TAD_BODY_PROGRAM = 7   /* inner and outer function given as postfix programs (tad_op), 1..TAD_MAX_ARGS operands;
                              their derivatives are derived by reverse accumulation (Sec. 2) at plan time */
} tad_body;

/*
 * Scalar functions given as postfix (reverse Polish) programs.  The inner program combines the operand values
 * of one extended index (TAD_OP_ARG p pushes the value of operand p), the outer program maps the summed inner
 * values to f (TAD_OP_SUM pushes that sum); each must leave exactly one value on the stack.  The outer program
 * may also read operands (Sec. 5.2: the function applied to the sum takes further tensors indexed by the
 * function index), but only those whose index matrix has zero columns for every summation index, so that they
 * have one value per function index; such an operand's gradient gets the additional term df * d outer / d x.
 */
typedef enum {
    TAD_OP_CONST = 0, /* push `value` */
    TAD_OP_ARG = 1,   /* push the value of operand `iarg` (outer program: see above) */
    TAD_OP_SUM = 2,   /* outer program only: push the summed inner value */
    TAD_OP_ADD = 3, TAD_OP_SUB = 4, TAD_OP_MUL = 5, TAD_OP_DIV = 6,   /* pop b, pop a, push a op b */
    TAD_OP_NEG = 7, TAD_OP_EXP = 8, TAD_OP_LOG = 9, TAD_OP_SIN = 10, TAD_OP_COS = 11, TAD_OP_TANH = 12,
    TAD_OP_SQRT = 13, /* pop a, push op(a) */
    TAD_OP_POWI = 14, /* pop a, push a^iarg for an integer exponent 1 <= iarg <= 16 */
    TAD_OP_STORE = 15, /* copy the top of the stack into temporary `iarg` (0 <= iarg < TAD_MAX_TEMPS); the stack is unchanged */
    TAD_OP_LOAD = 16   /* push temporary `iarg`, which an earlier operation of the same program has stored: a
                          sub-expression that is used several times is written once (Sec. 2: a node of the
                          expression graph may have several consumers) */
} tad_opcode;

typedef struct {
    int32_t op;    /* tad_opcode */
    int32_t iarg;  /* operand index (ARG), exponent (POWI) or temporary (STORE, LOAD) */
    double value;  /* CONST */
} tad_op;

#define TAD_MAX_PROGRAM 64 /* operations per program */
#define TAD_MAX_TEMPS 16   /* temporaries of TAD_OP_STORE / TAD_OP_LOAD per program */

/* Element-wise definition of f (Sec. 5.1): shape of f and the summation ranges Psi (Sec. 5.2). */
typedef struct {
    int32_t body;                  /* tad_body */
    int32_t n_f;                   /* number of function indices D_f (>= 1) */
    int64_t f_shape[TAD_MAX_EXT];  /* N^f */
    int32_t n_sum;                 /* number of summation indices; n_f + n_sum <= TAD_MAX_EXT */
    int64_t sum_lo[TAD_MAX_EXT];   /* inclusive constant limits of every summation index */
    int64_t sum_hi[TAD_MAX_EXT];
    /*
     * Extra linear conditions on the extended index [alpha k] (ranges of a sum that depend on other indices,
     * Sec. 5.2; the form that derived expressions have, Sec. 5.3): the term at [alpha k] is part of the sum iff
     *     sum_d constraint[j][d] * [alpha k]_d + constraint[j][n_f + n_sum] >= 0      for every j < n_constraints.
     * An expression with such conditions runs on the plan-driven generic kernels.
     */
    int32_t n_constraints;         /* 0..TAD_MAX_CONSTRAINTS */
    int64_t constraint[TAD_MAX_CONSTRAINTS][TAD_MAX_EXT + 1];
    /* TAD_BODY_PROGRAM only (ignored otherwise) */
    int32_t n_operands;            /* operands of the programs, 1..TAD_MAX_ARGS */
    int32_t n_inner, n_outer;      /* program lengths, 1..TAD_MAX_PROGRAM */
    tad_op inner[TAD_MAX_PROGRAM];
    tad_op outer[TAD_MAX_PROGRAM];
} tad_expr;

/*
 * One operand of the scalar body: a tensor x^p and its index map (Sec. 5.1; Sec. 5.2 for the extended map).
 * A tensor that occurs several times in the expression (Sec. 5.3: its gradient is the sum of the
 * contributions of all its occurrences) is given once as an operand of its own and then again, with
 * another index map, as operands whose `alias` names the first one.
 */
typedef struct {
    int32_t rank;                               /* D_p, 1..TAD_MAX_RANK */
    int64_t shape[TAD_MAX_RANK];                /* N^p */
    int32_t alias;                              /* 0: a tensor of its own; q + 1: a further occurrence of operand
                                                   q < p (itself not an alias; same rank and shape) */
    int64_t index[TAD_MAX_RANK][TAD_MAX_EXT];   /* A^p, D_p x (n_f + n_sum): argument index = A^p [alpha k] */
    int32_t needs_grad;                         /* derive a gather plan for this operand; for an alias the
                                                   flag of the operand it names is used */
} tad_arg;

/* plan flags */
#define TAD_PLAN_GENERIC_ONLY 1u /* never select a specialised kernel family; use the plan-driven generic kernels */
#define TAD_PLAN_DIRECT_FORM 2u  /* worked expression with a long summed index: evaluate the forward pass in the direct
                                    form sum_k (a_ik + b_jk)^2 on the vector ALUs instead of the expanded square on
                                    the matrix cores (for comparing the two forms; the gradients are not affected) */

#define TAD_PLAN_KEEP_PROGRAM 4u /* a program body that spells out one of the built-in bodies (same operations on the
                                    same operands; sums and products in either order, x * x for x^2) is normally planned
                                    as that body; with this flag it stays a program and runs on the interpreter kernels */

#define TAD_PLAN_NO_TERM_LISTS 8u /* a small expression (at most 1024 gradient elements and 1024 extended indices per
                                     gradient set in all, built-in body, plan-driven kernels) normally has the sets
                                     Gamma-hat(beta) of Sec. 5.1 that its ranges enumerate written out at plan time, and
                                     the device sums the listed terms; with this flag the device walks the ranges itself,
                                     as it does for every larger expression */

typedef struct tad_plan tad_plan; /* opaque, immutable after derivation, may be shared between threads */

/* What the derivation found for one argument (Sec. 4.1 quantities, host memory, row-major). */
typedef struct {
    int32_t rank;                                   /* R = rank of A^p */
    int32_t kernel_dim;                             /* kappa = (n_f + n_sum) - R */
    int32_t n_cokernel;                             /* D_p - R rows of C */
    int64_t smith[TAD_MAX_RANK];                    /* alpha_1..alpha_R, positive, alpha_i | alpha_{i+1} */
    int64_t U[TAD_MAX_RANK][TAD_MAX_RANK];          /* S = U A V, U is D_p x D_p */
    int64_t V[TAD_MAX_EXT][TAD_MAX_EXT];            /* V is (n_f+n_sum) x (n_f+n_sum) */
    int64_t K[TAD_MAX_EXT][TAD_MAX_KERNEL];         /* kernel basis, columns R.. of V */
    int64_t C[TAD_MAX_RANK][TAD_MAX_RANK];          /* cokernel rows, rows R.. of U */
    int32_t n_lower[TAD_MAX_KERNEL];                /* Fourier-Motzkin rows per kernel coordinate z_k */
    int32_t n_upper[TAD_MAX_KERNEL];
    int32_t n_feasibility;
    int32_t family;                                 /* kernel family chosen for this gradient (tad_family) */
    int32_t in_outer;                               /* 1 if the outer function reads this operand: its gradient has
                                                       the additional term df * d outer / d x */
    int32_t gather_layout;                          /* plan-driven (generic / program) kernels only: how the threads
                                                       are laid over this gradient: 0 one thread per element, 1 one
                                                       workgroup per element (long sums), 2 one thread per element
                                                       with the sum shared by workgroups (long sums read across the
                                                       contiguous direction of f) */
    int32_t gather_splits;                          /* ... and how many workgroups share one element (1: none) */
    int64_t gather_elements;                        /* ... and how many element numbers a launch runs over: all of
                                                       the tensor, or -- for a gradient that the cokernel or the
                                                       divisibility masks leave mostly zero -- only the box of the
                                                       transformed index y whose images beta = U^-1 [alpha y ; 0] are
                                                       the elements that pass those masks (Sec. 4.1) */
    int32_t listed;                                 /* 1: the terms of every element were listed at plan time (small
                                                       expression, see TAD_PLAN_NO_TERM_LISTS) */
} tad_plan_info;

typedef enum {
    TAD_FAMILY_GENERIC = 0,      /* one thread per gradient element, nested z loops (Sec. 5.1) */
    TAD_FAMILY_ROW_REDUCE = 1,   /* broadcast index: the whole last function dimension collapses */
    TAD_FAMILY_DIAGONAL = 2,     /* cokernel mask only, no summation */
    TAD_FAMILY_ANTIDIAGONAL = 3, /* one clipped window over x_{i+j} */
    TAD_FAMILY_WORKED = 4,       /* fused kernels for the worked expression */
    TAD_FAMILY_WORKED_MFMA = 5,  /* worked expression, long summed index: expanded cross term on MFMA */
    TAD_FAMILY_STRIDED = 6,      /* strided stencil */
    TAD_FAMILY_CONTRACTION = 7,  /* product of two matrices over one summation index: dense products on MFMA */
    TAD_FAMILY_PROGRAM = 8       /* program body: generic plan-driven kernels with an interpreter for the scalar part */
} tad_family;

/* which set of Fourier-Motzkin rows tad_plan_bound_row reads */
typedef enum { TAD_ROWS_LOWER = 0, TAD_ROWS_UPPER = 1, TAD_ROWS_FEASIBILITY = 2 } tad_row_kind;

/*
 * Derive the index plan of an expression (Sec. 5.3, the element-wise derivation
 * algorithm; index half only: the scalar partial derivatives of the built-in
 * bodies are fixed in the kernels).  Host only: touches no GPU.
 *   expr, args[n_args]  host, read; n_args must equal the body's operand count (aliases included)
 *   dt                  element type of every tensor
 *   flags               TAD_PLAN_* bits
 *   out                 receives a heap-allocated plan owned by the caller (tad_plan_free)
 * Errors: EINVAL (also: alias of a later operand or of another alias), ESHAPE (some [alpha k] that satisfies the
 * ranges and the extra conditions may map outside an argument -- decided on the rational relaxation, so
 * conservatively; alias with another rank or shape), EOVERFLOW, EUNSUPPORTED, ENOMEM.
 * An expression with aliases always runs on the plan-driven generic kernels.
 */
int tad_plan_derive(const tad_expr *expr, const tad_arg *args, int n_args, tad_dtype dt,
                    uint32_t flags, tad_plan **out);

void tad_plan_free(tad_plan *plan);

/* Bytes of device workspace tad_eval_forward / tad_eval_backward need: per-tile partial sums of the two-pass
 * reductions, intermediate tensors of the program bodies, and, on the plan-driven kernels, the partial sums of
 * gradient elements whose terms several workgroups share.  0 if the plan's kernels need none.
 * The paper's sketch of the gather form (Sec. 5.1, last paragraphs; Sec. 7) needs no temporary memory: one thread
 * sums all terms of one gradient element.  This library departs from that where a range collapses a whole
 * dimension: the terms of an element are split over a wavefront, a tile or several workgroups, and the partial
 * sums of the tiles wait here for a finishing pass that adds them in a fixed order. */
size_t tad_plan_workspace_bytes(const tad_plan *plan);

/*
 * Smith normal form parts and row counts for occurrence `occ` of the tensor given as operand `arg` (host,
 * written to *out): occ = 0 is operand `arg` itself, occ = k its k-th alias in operand order.
 * EINVAL if `arg` is an alias, has no plan, or has fewer occurrences.
 */
int tad_plan_query(const tad_plan *plan, int arg, int occ, tad_plan_info *out);

/*
 * One Fourier-Motzkin row (Sec. 4.2) for kernel coordinate `level` (0 = innermost z_1):
 *   lower:        scale * z_level >= coef_b . b(beta) + coef_z . z      (coef_z[m] = 0 for m <= level)
 *   upper:        scale * z_level <= coef_b . b(beta) + coef_z . z
 *   feasibility:  coef_b . b(beta) <= 0                                  (level ignored)
 * with b(beta) = [lo - I beta ; I beta - hi] (2 (n_f+n_sum) entries, Sec. 5.1 with zero-based box lo..hi).
 * coef_b has 2*TAD_MAX_EXT entries (entry j and TAD_MAX_EXT + j for index j), coef_z TAD_MAX_KERNEL. Host memory.
 * With extra conditions c_j . [alpha k] + c0_j >= 0 in the expression, b(beta) has one more entry per condition,
 * -c0_j - c_j . (I beta), and coef_c (TAD_MAX_CONSTRAINTS entries, may be NULL) receives its coefficients.
 */
int tad_plan_bound_row(const tad_plan *plan, int arg, int kind, int level, int row,
                       int64_t *scale, int64_t *coef_b, int64_t *coef_z, int64_t *coef_c);

/*
 * The set Gamma-hat(beta) of Sec. 5.2 -- all extended indices [alpha k] inside the ranges that the index map sends
 * to gradient element beta -- as the plan enumerates it (host): writes up to `cap` points ((n_f+n_sum) int64 each)
 * in lexicographic order to alpha_out and the total count to *n.  Uses exactly the masks (Sec. 4.1: cokernel,
 * divisibility), bound rows (Sec. 4.2) and index maps the kernels use, so comparing it with a scan of the whole
 * index box checks what the kernels sum over.
 */
int tad_plan_enumerate(const tad_plan *plan, int arg, int occ, const int64_t *beta,
                       int64_t *alpha_out, size_t cap, size_t *n);

/* |Gamma-hat(beta)| (Sec. 5.2) for every beta of operand `arg`, first occurrence only: the number of terms the
 * gather sum of that element has (host; counts has one int64 per element). */
int tad_plan_count_all(const tad_plan *plan, int arg, int64_t *counts);

/*
 * Forward evaluation of f (Sec. 5.1 / 5.2).  Enqueues kernels on `stream` (a hipStream_t, NULL = default
 * stream), never synchronises, never allocates.
 *   args_dev[n_args]  device, read; the entry of an alias operand is ignored (its tensor is the one it names)
 *   f_dev             device, overwritten (all of f)
 *   ws_dev, ws_bytes  device scratch of at least tad_plan_workspace_bytes (may be NULL if that is 0)
 */
int tad_eval_forward(const tad_plan *plan, const void *const *args_dev, void *f_dev,
                     void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Gather-form gradients (final formula of Sec. 5.1).
 *   f_dev     device, read: the forward result for the same args_dev
 *   df_dev    device, read: dl/df, shape of f
 *   dx_dev[p] device, overwritten with the full gradient in argument p's shape (zeros where the
 *             cokernel / divisibility / range conditions fail), summed over all occurrences of the tensor;
 *             NULL skips that gradient; must be NULL for an alias operand (EINVAL otherwise)
 * Same stream / workspace rules as tad_eval_forward.  Deterministic.
 */
int tad_eval_backward(const tad_plan *plan, const void *const *args_dev, const void *f_dev,
                      const void *df_dev, void *const *dx_dev, void *ws_dev, size_t ws_bytes,
                      void *stream);

/*
 * tad_eval_backward for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as tad_eval_backward
 * (bit-identical: the same kernels run), but the per-tile partial sums live in an array of
 * TAD_STATIC_SCRATCH_BYTES that is part of the library's device code: every GPU the library runs on holds one copy
 * until the process ends.  The call allocates nothing and frees nothing.
 *   - a plan with tad_plan_workspace_bytes above TAD_STATIC_SCRATCH_BYTES is refused with TAD_ENOMEM before
 *     anything is launched (the matrix-core family at 4096 x 4096 x 256 needs 64 MiB; the 8192 x 8192 x 5 worked
 *     expression 9.5 MiB);
 *   - the first call on a device looks up the array's address (no allocation); make it outside a stream capture;
 *   - all calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race on it and give wrong gradients; calls on one stream are ordered and safe.  The array keeps
 *     the last call's contents; the kernels overwrite every entry before reading it.
 * Errors: as tad_eval_backward; TAD_EDEVICE if the array's address cannot be obtained.
 */
#define TAD_STATIC_SCRATCH_BYTES (16u << 20)
int tad_eval_backward_static(const tad_plan *plan, const void *const *args_dev, const void *f_dev,
                             const void *df_dev, void *const *dx_dev, void *stream);

/*
 * The gradient of one occurrence of a tensor, written as element-wise defined tensors again (Sec. 5.3: a
 * derived expression has the form of the input expressions, with summation ranges that depend on the other
 * indices, so it can be evaluated, and differentiated once more, by the same machinery).  With
 * s_alpha = sum_k inner(...) and f_alpha = outer(s_alpha, operands at alpha) the gradient is
 *
 *     dx_beta = sum_z [conditions] g_{alpha(beta, z)} * (d inner / d x)(operand values at [alpha k](beta, z))   (part 0)
 *             + sum_z' [conditions] h_{alpha(beta, z')}                                                         (part 1)
 *     g_alpha = df_alpha * (d outer / d s)(s_alpha, ...),   h_alpha = df_alpha * (d outer / d x)(s_alpha, ...),
 *
 * part 1 only for an operand the outer function reads.  g and h contain the sum s_alpha, a second sum nested in
 * the first: they are expressions of their own over the function indices of the original one
 * (tad_plan_seed_expr), and the gradient is a small graph of expressions: evaluate the seed, then hand its
 * result to the derived expression as operand 0.  When the outer function is the identity g = df and no seed is
 * needed; when there is neither a summation nor a condition, outer(inner(x)) is treated as one function and
 * again no seed is needed.
 *
 * tad_plan_derived_expr, part 0.  Function indices of the new expression: beta (shape of the tensor); summation
 * indices: the kernel coordinates z with constant limits (their extremes over the box), and one more index t per
 * Smith divisor above 1 (the quotient (U beta)_r / alpha_r, tied to beta by the pair of conditions
 * (U beta)_r - alpha_r t >= 0 and <= 0: the divisibility mask written as a sum of at most one term);
 * conditions: the box rows of the original extended index [alpha k] = I beta + K z that those limits do not
 * already imply, the original extra conditions, and the cokernel rows C beta = 0 as pairs of inequalities.  Operand 0 is df or g
 * (shape of f); the others are those operands of the original expression that the partial derivative depends
 * on, in their original order (aliases stay aliases of one tensor).  The body is a program: inner = operand 0
 * times the symbolic partial derivative, outer = identity.
 * Part 1: the same construction from the operand's index map over the function indices alone; operand 0 is h,
 * there is no other operand, inner = operand 0.
 *   plan, arg, occ        as for tad_plan_query
 *   part                  0 or 1
 *   expr_out              host, written
 *   args_out              host, room for TAD_MAX_ARGS entries, written (needs_grad = 1 everywhere)
 *   operand_out           host, room for TAD_MAX_ARGS ints (may be NULL): operand_out[q] = operand of the original
 *                         expression that new operand q is; for operand 0: -1 = df itself, -2 = g (seed -1),
 *                         -3 - p = h of operand p (seed p)
 *   n_args_out            number of operands of the new expression
 * The outputs are written only on success.
 * Errors: EINVAL (as tad_plan_query; part 1 for an operand the outer function does not read); EUNSUPPORTED if the
 * result exceeds the limits of an expression (indices, operands, conditions, program length).
 *
 * tad_plan_seed_expr.  which = -1: g;  which = p: h of operand p (EINVAL unless the outer function reads p).
 * Same function indices, summation ranges and conditions as the original expression; operand 0 is df, operand
 * 1 + q is original operand q; inner = the original inner function, outer = operand 0 times the symbolic
 * derivative of the outer function.  EUNSUPPORTED if the original has TAD_MAX_ARGS operands already.
 */
int tad_plan_derived_expr(const tad_plan *plan, int arg, int occ, int part, tad_expr *expr_out, tad_arg *args_out,
                          int *operand_out, int *n_args_out);
int tad_plan_seed_expr(const tad_plan *plan, int which, tad_expr *expr_out, tad_arg *args_out, int *n_args_out);

/*
 * A gradient evaluated through its derived expressions (Sec. 5.3), end to end: the small graph described above --
 * seed expressions for g and h where the outer function is not the identity, part 0 of every occurrence of the
 * tensor, part 1 of the occurrences the outer function reads -- with a plan for each expression, evaluated by the
 * forward kernels, the parts added by the library in a fixed order.  The result equals what tad_eval_backward gives
 * for the same tensor (up to the order of the additions); nothing of the method is left to the caller.
 *
 * tad_derived_create   host only.  arg: an operand that is a tensor of its own (not an alias) and has a gradient
 *                      plan; all its occurrences are included.  The object is owned by the caller
 *                      (tad_derived_free), immutable, and independent of `plan` afterwards.
 *                      Errors: EINVAL, EUNSUPPORTED (an emitted expression exceeds the limits of tad_expr), EOVERFLOW, ENOMEM.
 * tad_derived_count    number of seed expressions and of parts in the graph (either pointer may be NULL).
 * tad_eval_derived     enqueues on `stream`, never synchronises, never allocates.
 *   args_dev[n_args]   device, read: the operands of the original expression (alias entries ignored)
 *   df_dev             device, read: dl/df
 *   dx_dev             device, overwritten with the gradient of tensor `arg`
 *   ws_dev, ws_bytes   device scratch of at least tad_derived_workspace_bytes: the seed tensors (shape of f), a second
 *                      tensor of the gradient's size when there are several parts, and the workspace of the
 *                      expressions' own kernels
 */
typedef struct tad_derived tad_derived;
int tad_derived_create(const tad_plan *plan, int arg, tad_derived **out);
void tad_derived_free(tad_derived *d);
size_t tad_derived_workspace_bytes(const tad_derived *d);
int tad_derived_count(const tad_derived *d, int *n_seeds, int *n_parts);
int tad_eval_derived(const tad_derived *d, const void *const *args_dev, const void *df_dev, void *dx_dev,
                     void *ws_dev, size_t ws_bytes, void *stream);

/* Name of the device kernel family used for the forward pass (tad_family). */
int tad_plan_forward_family(const tad_plan *plan);

/*
 * Host utilities of the integer machinery (Sec. 4), independent of any expression.
 *
 * tad_extended_gcd:       g = gcd(a, b) = a x + b y, g >= 0            (extended Euclidean algorithm)
 * tad_smith_normal_form:  S = U A V for the non-zero n x m matrix A (row-major, n, m <= 16); S is n x m,
 *                         U n x n, V m x m, all row-major host arrays owned by the caller; *rank = R.
 * tad_lattice_enumerate:  all integer x with A x = beta and lo <= x <= hi (inclusive), found through
 *                         Smith normal form and Fourier-Motzkin ranges (never by scanning the box), in
 *                         lexicographic order; n <= TAD_MAX_RANK, m <= TAD_MAX_EXT, kernel dimension
 *                         <= TAD_MAX_KERNEL.  Writes up to cap points (m int64 each), total to *count.
 */
/*
 * Host evaluation of the scalar functions of a TAD_BODY_PROGRAM plan in fp64, exactly the derived programs the
 * kernels interpret (for checking the symbolic differentiation without a GPU):
 *   which = -1: inner value            which = p >= 0: d inner / d operand p     (values[n_operands], host, read)
 *   which = -2: outer(sum, values)     which = -3: d outer / d sum               which = -4 - p: d outer / d operand p
 *   (the outer forms use `sum`, and `values` only if the outer program reads operands: it may be NULL otherwise)
 * Errors: EINVAL (not a program plan, bad `which`, NULL).
 */
int tad_plan_program_eval(const tad_plan *plan, int which, const double *values, double sum, double *out);
/*
 * Number of registers of the register form of one of those programs (`which` as above): the kernels read tensor
 * values, constants and the sum where an operation uses them, keep every other temporary in one of that many
 * vector registers per term and interpret several terms per pass (Sec. 2: the derivative is again a computational
 * graph; its live values decide the registers).  *registers_out = -1: more live values than the register form
 * holds; the kernels then interpret the form with one temporary per operation in the thread's private memory.
 * 0: the program is a single operand, a constant, or identically zero.
 * Errors: EINVAL (not a program plan, bad `which`, derivative not planned, NULL).
 */
int tad_plan_program_registers(const tad_plan *plan, int which, int *registers_out);

int tad_extended_gcd(int64_t a, int64_t b, int64_t *g, int64_t *x, int64_t *y);
int tad_smith_normal_form(const int64_t *A, int n, int m, int64_t *S, int64_t *U, int64_t *V, int *rank);
int tad_lattice_enumerate(const int64_t *A, int n, int m, const int64_t *lo, const int64_t *hi,
                          const int64_t *beta, int64_t *x_out, size_t cap, size_t *count);

/*
 * Instrumentation for benchmarks, not part of the evaluation path: time one kernel of the library with HIP events.  After tad_profile_begin(name, every)
 * each `every`-th launch of the kernel called `name` (the first one included, up to 4096 timed launches)
 * carries a start and a stop event attached to its own dispatch on the stream it is launched on, so the
 * pair reads that kernel's begin and end timestamps.  A timed launch delays the launch that follows it by
 * several microseconds; every > 1 spreads the samples over a run while keeping that cost small.
 * tad_profile_end waits for the events, returns the summed duration in milliseconds and the number of
 * timed launches, and switches the instrumentation off.  every < 1 is TAD_EINVAL.  Not thread safe against
 * concurrent evaluation calls from other threads while armed.
 */
int tad_profile_begin(const char *kernel_name, int every);
int tad_profile_end(double *total_ms, int *launches);

const char *tad_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TAD_H */
