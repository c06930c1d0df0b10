// Compact, trivially copyable form of an index plan as the kernels receive it
// (by value, as a kernel argument), and the mask / range evaluation shared by
// the device kernels and the host-side enumeration (tad_plan_enumerate).
//
// For gradient element beta of one argument (Sec. 4.1 / 5.1):
//   cokernel mask      C beta = 0
//   transformed index  y_r = (U beta)_r / alpha_r  (r < R), zero gradient unless every division is exact
//   function index     [alpha k] = V_R y + K z
//   ranges             scale * z_k >= (<=) k0 + ky . y + kz . z_{>k}      (Fourier-Motzkin rows with
//                      b(beta) = [lo - V_R y ; V_R y - hi] already substituted)
// Memory offsets of every tensor are linear in (y, z) because the index maps are linear.
#pragma once
#include <math.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define TAD_HD __host__ __device__ __forceinline__
#define TAD_UNROLL _Pragma("unroll")
#define TAD_NOUNROLL _Pragma("unroll 1")
#else
#define TAD_HD inline
#define TAD_UNROLL
#define TAD_NOUNROLL
#endif

#include "launch_geom.h"

namespace tad {

constexpr int kMaxExt = 6;
constexpr int kMaxRank = 4;
constexpr int kMaxArgs = 6;
constexpr int kMaxKernel = 4;
constexpr int kMaxCons = 8;
constexpr int kMaxRows = 32;   // lower + upper rows over all levels
constexpr int kMaxFeas = 12;
constexpr int kSlotF = kMaxArgs;        // offset slot of f / df
constexpr int kSlots = kMaxArgs + 1;

struct GRow {
    int32_t scale;
    int32_t k0;
    int32_t ky[kMaxRank];
    int32_t kz[kMaxKernel];
};

struct GatherPlan {
    int32_t rank;                 // D_p
    int32_t shape[kMaxRank];      // N^p
    int32_t R, kappa, nC, nF;
    int32_t U[kMaxRank][kMaxRank];   // first R rows of U
    int32_t diag[kMaxRank];          // alpha_1..alpha_R
    int32_t C[kMaxRank][kMaxRank];   // cokernel rows
    GRow feas[kMaxFeas];             // k0 + ky . y <= 0
    uint8_t lo_begin[kMaxKernel], lo_end[kMaxKernel];
    uint8_t hi_begin[kMaxKernel], hi_end[kMaxKernel];
    GRow rows[kMaxRows];
    int64_t offY[kSlots][kMaxRank];    // element offset of tensor slot s = offY[s] . y + offZ[s] . z
    int64_t offZ[kSlots][kMaxKernel];
    // masked gradients with few non-zero elements (live != 0): the elements that pass the masks are
    // beta = B y for the integer y of the box y_lo <= y < y_lo + y_n (some of them outside the tensor)
    int32_t live, live_count;          // live_count: points of the box
    int32_t y_lo[kMaxRank], y_n[kMaxRank];
    int32_t B[kMaxRank][kMaxRank];
};

// How the fallback gather kernels lay their threads over one gradient (decided on the host, per operand):
//   threads  one thread per element;
//   blocks   one block per element (long sums): the threads share the terms, taking the values of the innermost
//            kernel coordinate in turn -- coalesced when f is contiguous along that coordinate;
//   lanes    one thread per element again, chosen for long sums when f is contiguous along the ELEMENTS instead
//            (a column sum: neighbouring elements read neighbouring f, successive terms lie a row apart).
// For blocks and lanes, `splits` groups of threads can share an element (few elements or few blocks otherwise):
// fp64 partial sums in the workspace, added in a fixed order by a finishing kernel.
// Elements a launch over the gradient of this plan runs over: all of the tensor, or the box of y (live plans).
inline long long gather_launch_count(const GatherPlan &P, long long n_elements) { return P.live ? P.live_count : n_elements; }

enum GatherLayout { kLayoutThreads = 0, kLayoutBlocks = 1, kLayoutLanes = 2 };
struct GatherShape {
    int layout;
    int splits;
};
inline GatherShape gather_shape(const GatherPlan &P, long long n_elements, double terms_total) {
    GatherShape g{kLayoutThreads, 1};
    if (!use_cooperative_gather(n_elements, terms_total)) return g;
    g.layout = kLayoutBlocks;
    g.splits = cooperative_splits(n_elements, terms_total);
    if (P.kappa < 1 || P.rank < 1) return g;
    // offset of f between neighbouring elements (last index of beta) and between neighbouring values of z_0
    int64_t along_elements = 0;
    for (int r = 0; r < P.R; ++r) {
        const int64_t num = P.offY[kSlotF][r] * (int64_t)P.U[r][P.rank - 1];
        if (num % P.diag[r] != 0) return g;
        along_elements += num / P.diag[r];
    }
    const int64_t along_z = P.offZ[kSlotF][0];
    if ((along_elements < -1 || along_elements > 1) || (along_z > -16 && along_z < 16)) return g;
    g.layout = kLayoutLanes;
    const long long blocks = (n_elements + 255) / 256;
    const long long want = (2048 + blocks - 1) / blocks;                                  // about 2048 blocks in all
    const long long most = (long long)(terms_total / (double)n_elements / 256.0);         // at least 256 terms each
    long long sp = want < most ? want : most;
    if (sp > 256) sp = 256;
    g.splits = sp < 1 ? 1 : (int)sp;
    return g;
}

// Small expressions: the extended indices of every gradient element, which the ranges of the plan enumerate
// (the sets Gamma-hat(beta) of Sec. 5.1), written out on the host as element offsets into the tensors.  A launch
// over a few dozen elements with a handful of terms each is as long as the code it walks through, not as its
// arithmetic: with the terms listed that path is a few dozen instructions.
constexpr int kListElements = 1024;   // gradient elements of all operands together
constexpr int kListTerms = 1024;      // terms of all of them together
constexpr int kListSlots = 5;         // offsets per term: up to four operands, then f (and df)
struct TermList {
    int32_t n_grad;
    int32_t first_element[kMaxArgs + 1];   // gradient g owns the element numbers first_element[g] .. first_element[g + 1] - 1
    int32_t operand[kMaxArgs];             // whose gradient g is
    uint16_t first_term[kListElements + 1];   // element e sums the terms first_term[e] .. first_term[e + 1] - 1
    int32_t off[kListTerms][kListSlots];
};

struct ForwardPlan {
    int32_t n_f, n_sum;
    int32_t f_shape[kMaxExt];
    int32_t sum_lo[kMaxExt];
    int32_t sum_n[kMaxExt];            // number of values of each summation index
    int64_t off[kMaxArgs][kMaxExt];    // element offset of argument p = off[p] . [alpha k]
    int64_t base0[kMaxArgs];           // its part from the lower summation limits: sum_s off[p][n_f + s] * sum_lo[s]
    int64_t last_stride[kMaxArgs];     // off[p][n_f + n_sum - 1]: advance along the last summation index (0 without sums)
    int32_t n_cons;                    // extra conditions: cons[j] . [alpha k] + cons[j][n_f + n_sum] >= 0
    int32_t cons[kMaxCons][kMaxExt + 1];
};

// Scalar function in three-address form, as the kernels interpret it: operation i computes temporary i from
// earlier temporaries a[i], b[i] (or an operand / the sum / a constant).  Produced on the host from the user's
// postfix program or from its symbolic derivative (program.hpp).
constexpr int kMaxProgOps = 64;
constexpr int kMaxProgConst = 8;
enum ProgOp : uint8_t {
    P_CONST, P_ARG, P_SUM, P_ADD, P_SUB, P_MUL, P_DIV, P_NEG, P_EXP, P_LOG, P_SIN, P_COS, P_TANH, P_SQRT, P_POWI
};
constexpr int kProgRegs = 16;   // registers of the register form of a program
// operand codes of the register form: 0 .. kProgRegs-1 a register, then
constexpr int kCodeArg = 16;     // + p: the value of tensor operand p
constexpr int kCodeConst = 32;   // + c: constant c
constexpr int kCodeSum = 48;     // the sum (outer programs)
struct DevProg {
    int32_t n;        // operations
    int32_t result;   // temporary holding the result; -1: the function is identically zero
    uint8_t op[kMaxProgOps], a[kMaxProgOps], b[kMaxProgOps];   // a: first input / operand index / constant index / exponent base
    int8_t k[kMaxProgOps];                                     // exponent of P_POWI
    double cst[kMaxProgConst];
    // Register form of the same program, as the kernels' interpreter runs it: operands (tensor values, the sum,
    // constants) are read where they are used instead of being copied by operations of their own, and every other
    // temporary is assigned one of kProgRegs registers by its live range, so that the temporaries stay in vector
    // registers (indexed by a wave-uniform number) instead of the thread's private memory.
    //   word[i] = op | first << 8 | second << 16 | destination << 24        (n_words of them)
    //   first, second: an operand code (prog_code_*: register, tensor operand, constant, the sum); for P_POWI
    //   `second` is the exponent; destination: a register.  result_code: operand code of the result.
    // n_regs < 0: the program needs more registers than there are; only the form above exists.
    int32_t n_regs;
    int32_t n_words;
    int32_t result_code;
    uint32_t word[kMaxProgOps];
};

// Extra conditions of the expression at the extended index (function part ext[0..n_f), summation counters k).
TAD_HD bool forward_conditions(const ForwardPlan &P, const int32_t *ext, const int32_t *k) {
    bool ok = true;
    for (int e = 0; e < P.n_cons; ++e) {
        int32_t v = P.cons[e][P.n_f + P.n_sum];
        for (int d = 0; d < P.n_f; ++d) v += P.cons[e][d] * ext[d];
        for (int s = 0; s < P.n_sum; ++s) v += P.cons[e][P.n_f + s] * (P.sum_lo[s] + k[s]);
        ok = ok && v >= 0;
    }
    return ok;
}

// floor(a / b) and ceil(a / b) for b > 0, exact for negative a.  Divisors 1 and 2 (unit and stride-2
// index maps) avoid the integer division, which costs tens of instructions on the GPU.
TAD_HD int32_t floor_div_i(int32_t a, int32_t b) {
    if (b == 1) return a;
    if (b == 2) return a >> 1;
    int32_t q = a / b, r = a % b;
    return (r < 0) ? q - 1 : q;
}
TAD_HD int32_t ceil_div_i(int32_t a, int32_t b) {
    if (b == 1) return a;
    if (b == 2) return -((-a) >> 1);
    int32_t q = a / b, r = a % b;
    return (r > 0) ? q + 1 : q;
}

// Masks and transformed index for one beta.  Returns false when the gradient element is zero
// because of the cokernel condition, the divisibility condition or an infeasible range system.
TAD_HD bool gather_prepare(const GatherPlan &P, const int32_t *beta, int32_t *y) {
    for (int c = 0; c < P.nC; ++c) {
        int32_t s = 0;
        for (int d = 0; d < P.rank; ++d) s += P.C[c][d] * beta[d];
        if (s != 0) return false;
    }
    for (int r = 0; r < P.R; ++r) {
        int32_t s = 0;
        for (int d = 0; d < P.rank; ++d) s += P.U[r][d] * beta[d];
        if (P.diag[r] != 1) {
            if (s % P.diag[r] != 0) return false;
            s /= P.diag[r];
        }
        y[r] = s;
    }
    for (int f = 0; f < P.nF; ++f) {
        int32_t s = P.feas[f].k0;
        for (int r = 0; r < P.R; ++r) s += P.feas[f].ky[r] * y[r];
        if (s > 0) return false;
    }
    return true;
}

// Element number `idx` of a launch over one gradient -> position `lin` of the element in its tensor and its
// transformed index y.  The launch runs over all beta (idx = lin) or, for a plan with live != 0, over the box of
// y.  False: the element is zero by a mask, or (live plans) the point is no element at all: *lin < 0 then.
TAD_HD bool gather_element_index(const GatherPlan &P, int idx, int *lin, int32_t *y) {
    int32_t beta[kMaxRank];
    if (!P.live) {
        *lin = idx;
        int t = idx;
        for (int r = P.rank - 1; r >= 1; --r) { beta[r] = t % P.shape[r]; t /= P.shape[r]; }
        beta[0] = t;   // idx is below the number of elements: no division for the first index
        return gather_prepare(P, beta, y);
    }
    *lin = -1;
    int t = idx;
    for (int r = P.R - 1; r >= 0; --r) { y[r] = P.y_lo[r] + t % P.y_n[r]; t /= P.y_n[r]; }
    int pos = 0;
    for (int d = 0; d < P.rank; ++d) {
        int32_t b = 0;
        for (int r = 0; r < P.R; ++r) b += P.B[d][r] * y[r];
        if (b < 0 || b >= P.shape[d]) return false;
        pos = pos * P.shape[d] + b;
    }
    for (int f = 0; f < P.nF; ++f) {
        int32_t s = P.feas[f].k0;
        for (int r = 0; r < P.R; ++r) s += P.feas[f].ky[r] * y[r];
        if (s > 0) return false;   // the element exists and is zero: the launch has cleared it
    }
    *lin = pos;
    return true;
}

TAD_HD int32_t row_rhs(const GatherPlan &P, const GRow &g, int level, const int32_t *y, const int32_t *z) {
    int32_t s = g.k0;
    for (int r = 0; r < P.R; ++r) s += g.ky[r] * y[r];
    for (int m = level + 1; m < P.kappa; ++m) s += g.kz[m] * z[m];
    return s;
}

// Inclusive range of z_level given y and the outer coordinates z_{>level} (may be empty: lo > hi).
TAD_HD void gather_bounds(const GatherPlan &P, int level, const int32_t *y, const int32_t *z,
                          int32_t &lo, int32_t &hi) {
    int32_t l = INT32_MIN, h = INT32_MAX;
    for (int i = P.lo_begin[level]; i < P.lo_end[level]; ++i) {
        int32_t v = ceil_div_i(row_rhs(P, P.rows[i], level, y, z), P.rows[i].scale);
        l = v > l ? v : l;
    }
    for (int i = P.hi_begin[level]; i < P.hi_end[level]; ++i) {
        int32_t v = floor_div_i(row_rhs(P, P.rows[i], level, y, z), P.rows[i].scale);
        h = v < h ? v : h;
    }
    lo = l;
    hi = h;
}

// Fixed-size, loop-free form of the mask and range rows for plans whose ranges do not depend on outer
// kernel coordinates.  Evaluating the general form costs one dependent scalar load per row entry; this
// form is fetched with a few wide scalar loads and evaluated as straight-line code.  Unused rows hold
// neutral values, so no row counts are needed.
constexpr int kFlatRows = 3;
constexpr int kFlatFeas = 6;
constexpr int kFlatY = 3;

struct FlatLevel {
    int32_t ls[kFlatRows], lk0[kFlatRows], lky[kFlatRows][kFlatY];   // ls * z >= lk0 + lky . y
    int32_t hs[kFlatRows], hk0[kFlatRows], hky[kFlatRows][kFlatY];   // hs * z <= hk0 + hky . y
    float lrs[kFlatRows], hrs[kFlatRows];                            // 1 / ls, 1 / hs
};
constexpr int32_t kFlatNeutralLo = -(1 << 23) + 1, kFlatNeutralHi = (1 << 23) - 1;

struct FlatFeas {
    int32_t k0[kFlatFeas], ky[kFlatFeas][kFlatY];                    // k0 + ky . y <= 0
};

// 24-bit multiply (full rate on the GPU, a 32-bit integer multiply is quarter rate); flatten_level /
// flatten_feas only accept plans whose coefficients and index extents stay below 2^23.
TAD_HD int32_t mul24(int32_t a, int32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __mul24(a, b);
#else
    return a * b;
#endif
}

// floor(a / s) for s > 0 and |a| < 2^23 (guaranteed by flatten_level) without an integer division:
// a converts exactly, the float quotient a * (1 / s) is within 1/2 of a / s, so its floor is off by at most one
// and one correction in each direction makes it exact.
// The division itself, without the shortcuts for the divisors 1 and 2: straight-line code for kernels whose
// instruction footprint matters more than a few arithmetic instructions.
TAD_HD int32_t floor_div_float(int32_t a, int32_t s, float rs) {
    int32_t q = (int32_t)floorf((float)a * rs);
    const int32_t r = a - mul24(q, s);
    q += (r >= s) ? 1 : 0;
    q -= (r < 0) ? 1 : 0;
    return q;
}
TAD_HD int32_t floor_div_flat(int32_t a, int32_t s, float rs) {
    // a power of two (unit index maps, strides 2, 4, ...): an arithmetic shift is the exact floor, and the test is a
    // scalar one, uniform over the wave and far cheaper than the arithmetic below
    if ((s & (s - 1)) == 0) return a >> __builtin_ctz((unsigned)s);
    return floor_div_float(a, s, rs);
}

TAD_HD void flat_bounds(const FlatLevel &L, const int32_t *y, int32_t &lo, int32_t &hi) {
    int32_t l = INT32_MIN, h = INT32_MAX;
TAD_UNROLL
    for (int r = 0; r < kFlatRows; ++r) {
        int32_t a = L.lk0[r], b = L.hk0[r];
TAD_UNROLL
        for (int c = 0; c < kFlatY; ++c) {
            a += mul24(L.lky[r][c], y[c]);
            b += mul24(L.hky[r][c], y[c]);
        }
        a = -floor_div_flat(-a, L.ls[r], L.lrs[r]);   // ceil
        b = floor_div_flat(b, L.hs[r], L.hrs[r]);
        l = a > l ? a : l;
        h = b < h ? b : h;
    }
    lo = l;
    hi = h;
}

TAD_HD bool flat_feasible(const FlatFeas &F, const int32_t *y) {
    bool ok = true;
TAD_UNROLL
    for (int r = 0; r < kFlatFeas; ++r) {
        int32_t s = F.k0[r];
TAD_UNROLL
        for (int c = 0; c < kFlatY; ++c) s += mul24(F.ky[r][c], y[c]);
        ok = ok && s <= 0;
    }
    return ok;
}

TAD_HD int64_t gather_offset(const GatherPlan &P, int slot, const int32_t *y, const int32_t *z) {
    int64_t o = 0;
    for (int r = 0; r < P.R; ++r) o += P.offY[slot][r] * (int64_t)y[r];
    for (int m = 0; m < P.kappa; ++m) o += P.offZ[slot][m] * (int64_t)z[m];
    return o;
}

}  // namespace tad
