// Plan-driven kernels for scalar bodies given as programs.  Index handling is that of the generic kernels (one
// thread per function index / per gradient element, masks and nested ranges from the plan); the scalar part is a
// small interpreter of the three-address programs derived on the host: the inner and outer function for the
// forward pass, and for the backward pass their derivatives obtained by reverse accumulation (Sec. 2).
//
//   forward   f_alpha = outer( s_alpha, operands at alpha ),  s_alpha = sum_k inner(values at [alpha k])
//             (Sec. 5.2: the outer function may read operands whose index ignores the summation indices)
//   prepare   g_alpha = df_alpha * (d outer / d s)(s_alpha, ...)      (shared by all gradients, Sec. 5.3: the
//             derivative graph reuses common sub-expressions; stored in the workspace, and so is s_alpha if the
//             outer function reads operands)
//   gather    dx^p_beta = sum_{z in Sigma(beta)} g_alpha * (d inner / d x^p)(values at [alpha k]),  [alpha k] = I beta + K z
//   gather, operands of the outer function: dx^p_beta += sum over the alpha with A^p alpha = beta of
//             df_alpha * (d outer / d x^p)(s_alpha, operands at alpha), from the operand's plan over alpha alone
#include <hip/hip_runtime.h>

#include "gather_loop.h"
#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "launch_geom.h"

namespace tad {

template <typename T> struct Fn;
template <> struct Fn<float> {
    static __device__ __forceinline__ float exp_(float x) { return expf(x); }
    static __device__ __forceinline__ float log_(float x) { return logf(x); }
    static __device__ __forceinline__ float sin_(float x) { return sinf(x); }
    static __device__ __forceinline__ float cos_(float x) { return cosf(x); }
    static __device__ __forceinline__ float tanh_(float x) { return tanhf(x); }
    static __device__ __forceinline__ float sqrt_(float x) { return sqrtf(x); }
};
template <> struct Fn<double> {
    static __device__ __forceinline__ double exp_(double x) { return exp(x); }
    static __device__ __forceinline__ double log_(double x) { return log(x); }
    static __device__ __forceinline__ double sin_(double x) { return sin(x); }
    static __device__ __forceinline__ double cos_(double x) { return cos(x); }
    static __device__ __forceinline__ double tanh_(double x) { return tanh(x); }
    static __device__ __forceinline__ double sqrt_(double x) { return sqrt(x); }
};

template <typename T>
__device__ __forceinline__ T prog_unary(int op, T x, int k) {
    switch (op) {
    case P_NEG: return -x;
    case P_EXP: return Fn<T>::exp_(x);
    case P_LOG: return Fn<T>::log_(x);
    case P_SIN: return Fn<T>::sin_(x);
    case P_COS: return Fn<T>::cos_(x);
    case P_TANH: return Fn<T>::tanh_(x);
    case P_SQRT: return Fn<T>::sqrt_(x);
    case P_POWI: {
        T r = x;
        for (int e = 1; e < k; ++e) r *= x;
        return r;
    }
    default: return T(0);
    }
}

// One pass over the operations of the form with one temporary per operation; the temporaries live in the
// thread's private memory (programs whose live values do not fit the register form).
template <typename T>
__device__ __forceinline__ T prog_eval_temporaries(const DevProg &P, const T *v, T s) {
    T t[kMaxProgOps];
    for (int i = 0; i < P.n; ++i) {
        const int a = P.a[i], b = P.b[i];
        T r;
        switch (P.op[i]) {
        case P_CONST: r = (T)P.cst[a]; break;
        case P_ARG: r = v[a]; break;
        case P_SUM: r = s; break;
        case P_ADD: r = t[a] + t[b]; break;
        case P_SUB: r = t[a] - t[b]; break;
        case P_MUL: r = t[a] * t[b]; break;
        case P_DIV: r = t[a] / t[b]; break;
        default: r = prog_unary<T>(P.op[i], t[a], P.k[i]);
        }
        t[i] = r;
    }
    return t[P.result];
}

// The register form, for U terms at once: kProgRegs values per term in vector registers, addressed by the
// wave-uniform register numbers of the operation words (every lane runs the same program, so the words are
// scalar loads from the kernel arguments; the next word is fetched while the current operation runs).  Fetching
// and decoding an operation costs more than carrying it out: U terms share that cost.  One array per term: an
// array of kProgRegs values indexed by a uniform number stays in registers, a two-dimensional one does not.
template <typename T> struct ProgWidth { static constexpr int U = sizeof(T) == 4 ? 4 : 2; };   // terms per pass

// REGS chooses the form at compile time: a kernel holds one of the two, so that the kernels of the register
// form need no private memory at all (the runtime sets private memory up per launch, and slowly once a kernel asks
// for much of it).  The kernels below are built in three forms (template parameter FORM): 0 one temporary per
// operation, one term per pass; 1 registers, one term per pass (elements with one or two terms: several terms per
// pass would only cost registers, i.e. waves per SIMD); 2 registers, ProgWidth<T>::U terms per pass.
template <typename T, int U, bool REGS>
__device__ __forceinline__ void prog_eval_block(const DevProg &P, const T (&v)[kMaxArgs][U], const T (&s)[U], T (&out)[U]) {
    static_assert(U >= 1 && U <= 4, "one register array per term below");
    if (P.result < 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) out[u] = T(0);
        return;
    }
    if (!REGS) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            T col[kMaxArgs];
#pragma unroll
            for (int q = 0; q < kMaxArgs; ++q) col[q] = v[q][u];
            out[u] = prog_eval_temporaries<T>(P, col, s[u]);
        }
        return;
    }
    // not cleared: the allocation on the host writes every register before it is read
    T r0[kProgRegs], r1[kProgRegs], r2[kProgRegs], r3[kProgRegs];
    // DST[u] = EXPR for every term u; EXPR sees the term's register array as `r` and its number as `u`
#define TAD_EACH_TERM(DST, EXPR)                                                                    \
    {                                                                                               \
        { T(&r)[kProgRegs] = r0; constexpr int u = 0; (void)r; (void)u; DST[u] = EXPR; }            \
        if (U > 1) { T(&r)[kProgRegs] = r1; constexpr int u = U > 1 ? 1 : 0; (void)r; (void)u; DST[u] = EXPR; } \
        if (U > 2) { T(&r)[kProgRegs] = r2; constexpr int u = U > 2 ? 2 : 0; (void)r; (void)u; DST[u] = EXPR; } \
        if (U > 3) { T(&r)[kProgRegs] = r3; constexpr int u = U > 3 ? 3 : 0; (void)r; (void)u; DST[u] = EXPR; } \
    }
    // DST[u] = the operand with code CODE (wave-uniform): a register, a tensor operand, a constant or the sum.
    // The operand number selects code, not an address: v stays in registers.
#define TAD_FETCH(DST, CODE)                                                         \
    {                                                                                \
        static_assert(kMaxArgs == 6, "one case per operand");                        \
        const int code_ = (CODE);                                                    \
        if (code_ < kCodeArg) {                                                      \
            const int reg_ = code_ & (kProgRegs - 1);                                \
            TAD_EACH_TERM(DST, r[reg_])                                              \
        } else if (code_ < kCodeConst) {                                             \
            switch (code_ - kCodeArg) {                                              \
            case 0: TAD_EACH_TERM(DST, v[0][u]) break;                               \
            case 1: TAD_EACH_TERM(DST, v[1][u]) break;                               \
            case 2: TAD_EACH_TERM(DST, v[2][u]) break;                               \
            case 3: TAD_EACH_TERM(DST, v[3][u]) break;                               \
            case 4: TAD_EACH_TERM(DST, v[4][u]) break;                               \
            default: TAD_EACH_TERM(DST, v[5][u])                                     \
            }                                                                        \
        } else if (code_ < kCodeSum) {                                               \
            const T cst_ = (T)P.cst[(code_ - kCodeConst) & (kMaxProgConst - 1)];     \
            TAD_EACH_TERM(DST, cst_)                                                 \
        } else {                                                                     \
            TAD_EACH_TERM(DST, s[u])                                                 \
        }                                                                            \
    }
    uint32_t w = P.word[0];
    for (int i = 0; i < P.n_words; ++i) {
        const uint32_t next = P.word[(i + 1) & (kMaxProgOps - 1)];
        const int op = (int)(w & 0xff), first = (int)((w >> 8) & 0xff), second = (int)((w >> 16) & 0xff);
        const int dst = (int)(w >> 24) & (kProgRegs - 1);
        T x[U], y[U], o[U];
        TAD_FETCH(x, first)
        if (op >= P_ADD && op <= P_DIV) TAD_FETCH(y, second)
        switch (op) {
        case P_ADD:
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = x[u] + y[u];
            break;
        case P_SUB:
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = x[u] - y[u];
            break;
        case P_MUL:
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = x[u] * y[u];
            break;
        case P_DIV:
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = x[u] / y[u];
            break;
        default:
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = prog_unary<T>(op, x[u], second);
        }
        r0[dst] = o[0];
        if (U > 1) r1[dst] = o[U > 1 ? 1 : 0];
        if (U > 2) r2[dst] = o[U > 2 ? 2 : 0];
        if (U > 3) r3[dst] = o[U > 3 ? 3 : 0];
        w = next;
    }
    TAD_FETCH(out, P.result_code)
#undef TAD_FETCH
#undef TAD_EACH_TERM
}

// one term
template <typename T, int FORM>
__device__ __forceinline__ T prog_eval(const DevProg &P, const T *v, T s) {
    T vv[kMaxArgs][1], ss[1] = {s}, out[1];
#pragma unroll
    for (int q = 0; q < kMaxArgs; ++q) vv[q][0] = v[q];
    prog_eval_block<T, 1, (FORM > 0)>(P, vv, ss, out);
    return out[0];
}

// A run of `n` terms whose operand q advances by stp[q] elements per term from ptr[q] (null: the program does
// not read it), weighted by *wp (advancing by ws; null: weight 1) and with the sum operand read from *sp (same
// stride; null: 0): ProgWidth<T>::U terms per pass of the interpreter, added in ascending order.  The terms past
// the end of the last pass repeat the run's first term and are dropped.
template <typename T, int FORM>
__device__ __forceinline__ double prog_run(const DevProg &P, const T *const (&ptr0)[kMaxArgs], const int64_t (&stp)[kMaxArgs],
                                           const T *wp, const T *sp, int64_t ws, int32_t n, double acc) {
    constexpr int U = FORM == 2 ? ProgWidth<T>::U : 1;
    const T *ptr[kMaxArgs];
#pragma unroll
    for (int q = 0; q < kMaxArgs; ++q) ptr[q] = ptr0[q];
    for (int32_t it = 0; it < n; it += U) {
        T v[kMaxArgs][U], sv[U], wv[U], o[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t m = it + u < n ? u : -(int64_t)it;   // in steps from the current position
#pragma unroll
            for (int q = 0; q < kMaxArgs; ++q) v[q][u] = ptr[q] ? ptr[q][m * stp[q]] : T(0);
            sv[u] = sp ? sp[(it + m) * ws] : T(0);
            wv[u] = wp ? wp[(it + m) * ws] : T(1);
        }
        prog_eval_block<T, U, (FORM > 0)>(P, v, sv, o);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (it + u < n) acc += (double)(wv[u] * o[u]);
#pragma unroll
        for (int q = 0; q < kMaxArgs; ++q)
            if (ptr[q]) ptr[q] += (int64_t)U * stp[q];
    }
    return acc;
}

// sum over the summation box of inner(values) for one function index, fp64 accumulation; base[p] receives the
// offset of operand p at the first summation index (for an operand that ignores the summation indices: its
// offset at this function index)
// `parts` cooperating threads share the sum: thread `part` takes the terms part, part + parts, ... of the box
// in row-major order (last summation index fastest), so that a wavefront reads neighbouring elements together.
template <typename T, int FORM>
__device__ double inner_sum(const ForwardPlan &P, const DevProg &inner, int n_ops, const ArgPtrs &A, int lin,
                            int64_t *base, int part = 0, int parts = 1) {
    // unrolled to the largest rank and cut short by tests of the uniform rank: every field of the plan comes from a
    // fixed place in the kernel arguments (see forward_sum of the built-in bodies)
    int32_t ext[kMaxExt];
    {
        int t = lin;
#pragma unroll
        for (int d = kMaxExt - 1; d >= 1; --d) {
            ext[d] = 0;
            if (d < P.n_f) {
                const int s = P.f_shape[d], q = t / s;
                ext[d] = t - q * s;
                t = q;
            }
        }
        ext[0] = t;   // lin is below the number of function elements: no division for the first index
    }
#pragma unroll
    for (int p = 0; p < kMaxArgs; ++p) {
        if (p < n_ops) {
            int64_t o = P.base0[p];
#pragma unroll
            for (int d = 0; d < kMaxExt; ++d)
                if (d < P.n_f) o += P.off[p][d] * (int64_t)ext[d];
            base[p] = o;
        }
    }
    int32_t k[kMaxExt] = {0};
    double acc = 0.0;
    const int last = P.n_sum - 1;
    const int32_t n_last = last >= 0 ? P.sum_n[last] : 1;
    if (P.n_cons == 0 && last >= 0 && (parts == 1 || last == 0 || n_last >= parts)) {
        // no extra conditions: the innermost summation index is a run of n_last terms with constant strides;
        // cooperating threads take its terms in turn
        const T *bp[kMaxArgs];
        int64_t stp[kMaxArgs];
#pragma unroll
        for (int p = 0; p < kMaxArgs; ++p) {
            bp[p] = p < n_ops ? static_cast<const T *>(A.p[p]) + base[p] : nullptr;
            stp[p] = p < n_ops ? P.off[p][P.n_f + last] * parts : 0;
        }
        const int32_t mine = part < n_last ? (n_last - part + parts - 1) / parts : 0;
        for (;;) {
            const T *ptr[kMaxArgs];
#pragma unroll
            for (int p = 0; p < kMaxArgs; ++p) {
                int64_t o = 0;
                if (p < n_ops) {
#pragma unroll
                    for (int sidx = 0; sidx < kMaxExt; ++sidx)
                        if (sidx < last) o += P.off[p][P.n_f + sidx] * (int64_t)k[sidx];
                    o += P.off[p][P.n_f + last] * (int64_t)part;
                }
                ptr[p] = bp[p] ? bp[p] + o : nullptr;
            }
            acc = prog_run<T, FORM>(inner, ptr, stp, nullptr, nullptr, 0, mine, acc);
            int sidx = last - 1;
            for (; sidx >= 0; --sidx) {
                if (++k[sidx] < P.sum_n[sidx]) break;
                k[sidx] = 0;
            }
            if (sidx < 0) break;
        }
        return acc;
    }
    auto term = [&]() {
        if (forward_conditions(P, ext, k)) {   // a term outside the extra conditions is not part of the sum
            T v[kMaxArgs] = {};
            for (int p = 0; p < n_ops; ++p) {
                int64_t o = base[p];
                for (int s = 0; s < P.n_sum; ++s) o += P.off[p][P.n_f + s] * (int64_t)k[s];
                v[p] = static_cast<const T *>(A.p[p])[o];
            }
            acc += (double)prog_eval<T, FORM>(inner, v, T(0));
        }
    };
    if (parts > 1) {
        int64_t total = 1;
        for (int s = 0; s < P.n_sum; ++s) total *= P.sum_n[s];
        for (int64_t t = part; t < total; t += parts) {
            int64_t r = t;
            for (int s = P.n_sum - 1; s >= 0; --s) { k[s] = (int32_t)(r % P.sum_n[s]); r /= P.sum_n[s]; }
            term();
        }
        return acc;
    }
    for (;;) {
        term();
        int s = P.n_sum - 1;
        for (; s >= 0; --s) {
            if (++k[s] < P.sum_n[s]) break;
            k[s] = 0;
        }
        if (s < 0) break;
    }
    return acc;
}

// df == nullptr: out = outer(sum, operands) (forward);  otherwise out = df * (d outer / d sum)(sum, operands)
// (backward preparation).  outer_mask: operands `outer` reads.  s_out (may be null): receives the sum.
// (fp32: three wavefronts per SIMD -- the register forms would otherwise end a few registers above that step)
template <typename T, int FORM>
__global__ __launch_bounds__(256, sizeof(T) == 4 ? 3 : 1) void k_program_forward(const ForwardPlan P, const DevProg inner, const DevProg outer,
                                                         int n_ops, uint32_t outer_mask, const ArgPtrs A,
                                                         const T *__restrict__ df, T *__restrict__ out,
                                                         T *__restrict__ s_out, int nf) {
    const int lin = blockIdx.x * blockDim.x + threadIdx.x;
    if (lin >= nf) return;
    int64_t base[kMaxArgs];
    const T s = (T)inner_sum<T, FORM>(P, inner, n_ops, A, lin, base);
    T v[kMaxArgs] = {};
    for (int p = 0; p < n_ops; ++p) v[p] = ((outer_mask >> p) & 1u) ? static_cast<const T *>(A.p[p])[base[p]] : T(0);
    const T o = prog_eval<T, FORM>(outer, v, s);
    out[lin] = df ? df[lin] * o : o;
    if (s_out) s_out[lin] = s;
}

// the same with one block per function index (long sums): the 256 threads share the sum
template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_forward_coop(const ForwardPlan P, const DevProg inner, const DevProg outer,
                                                              int n_ops, uint32_t outer_mask, const ArgPtrs A,
                                                              const T *__restrict__ df, T *__restrict__ out,
                                                              T *__restrict__ s_out, double *__restrict__ partial) {
    // gridDim.y blocks share a function index (few function indices): their sums go to `partial` and
    // k_program_forward_finish applies the outer function
    __shared__ double red[4];
    const int lin = blockIdx.x;
    int64_t base[kMaxArgs];
    const double mine = inner_sum<T, FORM>(P, inner, n_ops, A, lin, base, (int)(blockIdx.y * 256 + threadIdx.x),
                                           (int)(256 * gridDim.y));
    const double total = block_sum_256(mine, red);
    if (threadIdx.x != 0) return;
    if (partial) {
        partial[(size_t)lin * gridDim.y + blockIdx.y] = total;
        return;
    }
    const T s = (T)total;
    T v[kMaxArgs] = {};
    for (int p = 0; p < n_ops; ++p) v[p] = ((outer_mask >> p) & 1u) ? static_cast<const T *>(A.p[p])[base[p]] : T(0);
    const T o = prog_eval<T, FORM>(outer, v, s);
    out[lin] = df ? df[lin] * o : o;
    if (s_out) s_out[lin] = s;
}

// Second pass of a forward sum shared by several blocks per function index: one wavefront per function index adds
// the partial sums (lane l the sums l, l + 64, ... in ascending order, then a fixed tree) and applies the outer
// function as k_program_forward does.
template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_forward_finish(const ForwardPlan P, const DevProg outer, int n_ops,
                                                                uint32_t outer_mask, const ArgPtrs A,
                                                                const T *__restrict__ df, T *__restrict__ out,
                                                                T *__restrict__ s_out, const double *__restrict__ partial,
                                                                int splits, int nf) {
    const int lin = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (lin >= nf) return;   // the whole wavefront leaves together
    double mine = 0.0;
    for (int sp = lane; sp < splits; sp += 64) mine += partial[(size_t)lin * splits + sp];
    const T s = (T)wave_sum_all(mine);
    if (lane != 0) return;
    int32_t ext[kMaxExt];
    {
        int t = lin;
        for (int d = P.n_f - 1; d >= 0; --d) { ext[d] = t % P.f_shape[d]; t /= P.f_shape[d]; }
    }
    T v[kMaxArgs] = {};
    for (int p = 0; p < n_ops; ++p) {
        if (!((outer_mask >> p) & 1u)) continue;
        int64_t o = 0;   // an operand of the outer function ignores the summation indices
        for (int d = 0; d < P.n_f; ++d) o += P.off[p][d] * (int64_t)ext[d];
        v[p] = static_cast<const T *>(A.p[p])[o];
    }
    const T o = prog_eval<T, FORM>(outer, v, s);
    out[lin] = df ? df[lin] * o : o;
    if (s_out) s_out[lin] = s;
}

// Term df * d outer / d x^p of element number `idx` of an operand the outer function reads: masks and ranges from
// the operand's plan over the function indices alone.
template <typename T, int FORM>
__device__ __forceinline__ bool outer_element(const GatherPlan &P, const DevProg &douter_p, int n_ops, uint32_t outer_mask,
                                              const ArgPtrs &A, const T *__restrict__ s_ws, const T *__restrict__ df,
                                              int idx, int *lin, int part, int parts, double *sum, int group = 0,
                                              int groups = 1) {
    int32_t y[kMaxRank] = {0, 0, 0, 0};
    *sum = 0.0;
    if (!gather_element_index(P, idx, lin, y)) return false;
    double acc = 0.0;
    gather_loops(P, y, part, parts, [&](const int32_t *z, int32_t n, int32_t step) {
        const T *ptr[kMaxArgs];
        int64_t stp[kMaxArgs];
#pragma unroll
        for (int q = 0; q < kMaxArgs; ++q) {
            const bool on = q < n_ops && ((outer_mask >> q) & 1u);
            ptr[q] = on ? static_cast<const T *>(A.p[q]) + gather_offset(P, q, y, z) : nullptr;
            stp[q] = on ? P.offZ[q][0] * step : 0;
        }
        const int64_t of = gather_offset(P, kSlotF, y, z);
        acc = prog_run<T, FORM>(douter_p, ptr, stp, df + of, s_ws + of, P.offZ[kSlotF][0] * step, n, acc);
    }, group, groups);
    *sum = acc;
    return true;
}

template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_gather_outer(const GatherPlan P, const DevProg douter_p, int n_ops,
                                                              uint32_t outer_mask, const ArgPtrs A,
                                                              const T *__restrict__ s_ws, const T *__restrict__ df,
                                                              T *__restrict__ dx, int n, int accumulate) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    double acc;
    int lin;
    const bool live = outer_element<T, FORM>(P, douter_p, n_ops, outer_mask, A, s_ws, df, idx, &lin, 0, 1, &acc);
    store_element(dx, lin, live, acc, accumulate);
}

// one block per gradient element (few elements, many function indices each)
template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_gather_outer_coop(const GatherPlan P, const DevProg douter_p, int n_ops,
                                                                   uint32_t outer_mask, const ArgPtrs A,
                                                                   const T *__restrict__ s_ws, const T *__restrict__ df,
                                                                   T *__restrict__ dx, int accumulate,
                                                                   double *__restrict__ partial, int32_t *__restrict__ live_out) {
    __shared__ double red[4];
    const int idx = blockIdx.x;
    double acc;
    int lin;
    const bool live = outer_element<T, FORM>(P, douter_p, n_ops, outer_mask, A, s_ws, df, idx, &lin,
                                             threadIdx.x, 256, &acc, (int)blockIdx.y, (int)gridDim.y);
    const double total = block_sum_256(acc, red);
    if (threadIdx.x != 0) return;
    if (partial) store_partial(partial, live_out, idx, lin, live, total);   // several blocks share the element
    else store_element(dx, lin, live, total, accumulate);
}

// Element number `idx` of the launch (gather_element_index: *lin receives its position in the tensor): masks, then
// the terms of the z loops shared by `parts` threads.
template <typename T, int FORM>
__device__ __forceinline__ bool program_element(const GatherPlan &P, const DevProg &dinner, int n_ops, const ArgPtrs &A,
                                                const T *__restrict__ g, int idx, int *lin, int part, int parts,
                                                double *sum, int group = 0, int groups = 1) {
    int32_t y[kMaxRank] = {0, 0, 0, 0};
    *sum = 0.0;
    if (!gather_element_index(P, idx, lin, y)) return false;
    double acc = 0.0;
    gather_loops(P, y, part, parts, [&](const int32_t *z, int32_t n, int32_t step) {
        const T *ptr[kMaxArgs];
        int64_t stp[kMaxArgs];
#pragma unroll
        for (int q = 0; q < kMaxArgs; ++q) {
            const bool on = q < n_ops;
            ptr[q] = on ? static_cast<const T *>(A.p[q]) + gather_offset(P, q, y, z) : nullptr;
            stp[q] = on ? P.offZ[q][0] * step : 0;
        }
        acc = prog_run<T, FORM>(dinner, ptr, stp, g + gather_offset(P, kSlotF, y, z), nullptr, P.offZ[kSlotF][0] * step, n, acc);
    }, group, groups);
    *sum = acc;
    return true;
}

template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_gather(const GatherPlan P, const DevProg dinner, int n_ops,
                                                        const ArgPtrs A, const T *__restrict__ g,
                                                        T *__restrict__ dx, int n, int accumulate, int classify) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x, lane = threadIdx.x & 63;
    const bool inside = idx < n;
    bool heavy = false;
    int lin = -1;
    if (classify && inside) {   // classify == 0: the whole expression has fewer terms than one heavy element would
        int32_t y[kMaxRank] = {0, 0, 0, 0};
        heavy = gather_element_index(P, idx, &lin, y) && gather_estimate(P, y) >= kHeavyTerms;
    }
    double acc = 0.0;
    bool live = false;
    if (inside && !heavy) live = program_element<T, FORM>(P, dinner, n_ops, A, g, idx, &lin, 0, 1, &acc);
    // an element with many terms is summed by the whole wavefront (the masks can leave few elements with all the work)
    for (unsigned long long todo = __ballot(heavy); todo; todo &= todo - 1) {
        const int src = __ffsll((long long)todo) - 1;
        double part_sum;
        int lin_src;
        program_element<T, FORM>(P, dinner, n_ops, A, g, __shfl(idx, src, 64), &lin_src, lane, 64, &part_sum);
        const double total = wave_sum_all(part_sum);
        if (lane == src) { acc = total; live = true; lin = lin_src; }
    }
    if (!inside) return;
    store_element(dx, lin, live, acc, accumulate);
}

// one block per gradient element (few elements, long sums)
template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_gather_coop(const GatherPlan P, const DevProg dinner, int n_ops,
                                                             const ArgPtrs A, const T *__restrict__ g,
                                                             T *__restrict__ dx, int accumulate,
                                                             double *__restrict__ partial, int32_t *__restrict__ live_out) {
    __shared__ double red[4];
    const int idx = blockIdx.x;
    double acc;
    int lin;
    const bool live = program_element<T, FORM>(P, dinner, n_ops, A, g, idx, &lin, threadIdx.x, 256, &acc,
                                               (int)blockIdx.y, (int)gridDim.y);
    const double total = block_sum_256(acc, red);
    if (threadIdx.x != 0) return;
    if (partial) store_partial(partial, live_out, idx, lin, live, total);   // several blocks share the element
    else store_element(dx, lin, live, total, accumulate);
}

// one thread per gradient element, the terms of every element shared by gridDim.y blocks (long sums read across
// the contiguous direction of g: neighbouring threads read neighbouring g)
template <typename T, int FORM>
__global__ __launch_bounds__(256) void k_program_gather_lanes(const GatherPlan P, const DevProg dinner, int n_ops,
                                                              const ArgPtrs A, const T *__restrict__ g,
                                                              T *__restrict__ dx, int n, int accumulate,
                                                              double *__restrict__ partial, int32_t *__restrict__ live_out) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    double acc;
    int lin;
    const bool live = program_element<T, FORM>(P, dinner, n_ops, A, g, idx, &lin, 0, 1, &acc, (int)blockIdx.y,
                                               (int)gridDim.y);
    if (partial) store_partial(partial, live_out, idx, lin, live, acc);
    else store_element(dx, lin, live, acc, accumulate);
}

// Several gradients of a small expression in one launch (every launch starts with cold instruction caches, which a
// wavefront that walks this code once pays dearly: together instead of one after the other).  Workgroups of one
// wavefront; workgroup b works on gradient g with first[g] <= b < first[g + 1].
struct MultiProgramGather {
    int32_t count;
    int32_t first[kMaxArgs + 1];
    int32_t n[kMaxArgs];         // elements of gradient g
    void *dx[kMaxArgs];
    GatherPlan plan[kMaxArgs];
    DevProg dinner[kMaxArgs];    // d inner / d operand of gradient g
};
template <typename T, int FORM>
__global__ __launch_bounds__(64) void k_program_gather_multi(const MultiProgramGather M, int n_ops, const ArgPtrs A,
                                                             const T *__restrict__ g) {
    int w = 0;
    while (w + 1 < M.count && (int)blockIdx.x >= M.first[w + 1]) ++w;   // the same for the whole workgroup
    const int idx = ((int)blockIdx.x - M.first[w]) * 64 + (int)threadIdx.x;
    if (idx >= M.n[w]) return;
    double acc;
    int lin;
    const bool live = program_element<T, FORM>(M.plan[w], M.dinner[w], n_ops, A, g, idx, &lin, 0, 1, &acc);
    store_element(static_cast<T *>(M.dx[w]), lin, live, acc, 0);
}

// a program that is identically zero is never interpreted
static bool has_register_form(const DevProg &P) { return P.result < 0 || P.n_regs >= 0; }

// Kernel form for a launch whose runs have about `run_terms` terms: several terms per pass pay from three terms on.
static int program_form(bool registers, double run_terms) { return !registers ? 0 : run_terms >= 3.0 ? 2 : 1; }

#define TAD_LAUNCH_FORM(form, name, kernel, ...)                             \
    do {                                                                     \
        switch (form) {                                                      \
        case 2: TAD_LAUNCH(name, (kernel<T, 2>), __VA_ARGS__); break;        \
        case 1: TAD_LAUNCH(name, (kernel<T, 1>), __VA_ARGS__); break;        \
        default: TAD_LAUNCH(name, (kernel<T, 0>), __VA_ARGS__);              \
        }                                                                    \
    } while (0)

template <typename T>
static int fwd_t(const tad_plan &pl, const void *const *args, const void *df, void *out, void *s_out, void *ws,
                 hipStream_t s) {
    ArgPtrs A{};
    for (size_t q = 0; q < pl.args.size(); ++q) A.p[q] = args[pl.root[q]];
    const int nf = (int)pl.f_count;
    const bool fwd_regs = has_register_form(pl.prog.inner) && has_register_form(df ? pl.prog.douter : pl.prog.outer);
    // the runs of the forward sum are the values of the last summation index
    const int form = program_form(fwd_regs, pl.fwd.n_sum > 0 ? (double)pl.fwd.sum_n[pl.fwd.n_sum - 1] : 1.0);
    if (use_cooperative_gather(nf, pl.terms_total)) {   // every function index sums many terms
        const int splits = cooperative_splits(nf, pl.terms_total);
        double *const partial = splits > 1 ? reinterpret_cast<double *>(static_cast<char *>(ws) + pl.split_ws_offset) : nullptr;
        TAD_LAUNCH_FORM(form, "k_program_forward_coop", k_program_forward_coop, dim3(nf, splits), dim3(256), 0, s, pl.fwd,
                        pl.prog.inner, df ? pl.prog.douter : pl.prog.outer, (int)pl.args.size(), pl.prog.outer_mask, A,
                        static_cast<const T *>(df), static_cast<T *>(out), static_cast<T *>(s_out), partial);
        if (splits > 1) {
            if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
            TAD_LAUNCH_FORM(form, "k_program_forward_finish", k_program_forward_finish, dim3((nf + 3) / 4), dim3(256), 0,
                            s, pl.fwd, df ? pl.prog.douter : pl.prog.outer, (int)pl.args.size(), pl.prog.outer_mask, A,
                            static_cast<const T *>(df), static_cast<T *>(out), static_cast<T *>(s_out),
                            (const double *)partial, splits, nf);
        }
    } else
        TAD_LAUNCH_FORM(form, "k_program_forward", k_program_forward, dim3((nf + 255) / 256), dim3(256), 0, s, pl.fwd,
                        pl.prog.inner, df ? pl.prog.douter : pl.prog.outer, (int)pl.args.size(), pl.prog.outer_mask, A,
                        static_cast<const T *>(df), static_cast<T *>(out), static_cast<T *>(s_out), nf);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

int program_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s) {
    return pl.dtype == TAD_F64 ? fwd_t<double>(pl, args, nullptr, f, nullptr, ws, s)
                               : fwd_t<float>(pl, args, nullptr, f, nullptr, ws, s);
}

template <typename T>
static int bwd_t(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                 hipStream_t s) {
    // workspace: g = df * (d outer / d sum), then (only if the outer function reads operands) the sums themselves
    T *const s_ws = pl.prog.outer_mask
                        ? reinterpret_cast<T *>(static_cast<char *>(ws) + align256((size_t)pl.f_count * sizeof(T)))
                        : nullptr;
    int rc = fwd_t<T>(pl, args, df, ws, s_ws, ws, s);
    if (rc) return rc;
    ArgPtrs A{};
    for (size_t q = 0; q < pl.args.size(); ++q) A.p[q] = args[pl.root[q]];
    const int n_ops = (int)pl.args.size();
    // partial sums of gradient elements shared by several blocks, and behind them one flag per element
    double *const split_partial = reinterpret_cast<double *>(static_cast<char *>(ws) + pl.split_ws_offset);
    auto split_live = [&](int n, int splits) {
        return reinterpret_cast<int32_t *>(reinterpret_cast<char *>(split_partial) + align256((size_t)n * splits * 8));
    };
    // a small expression without aliases whose outer function reads no operand: all gradients in one launch
    if (!pl.has_alias && !pl.prog.outer_mask && pl.terms_total < (double)kHeavyTerms) {
        MultiProgramGather M{};
        bool fits = true, registers = true;
        long long blocks = 0;
        for (size_t q = 0; q < pl.args.size() && fits; ++q) {
            if (!dx[q]) continue;
            const long long n = pl.arg_count[q];
            fits = pl.ap[q].derived && n <= (1 << 16) &&
                   gather_shape(pl.ap[q].dev, n, pl.terms_total).layout == kLayoutThreads;
            if (!fits) break;
            const int w = M.count++;
            M.first[w] = (int32_t)blocks;
            M.n[w] = (int32_t)n;
            M.dx[w] = dx[q];
            M.plan[w] = pl.ap[q].dev;
            M.plan[w].live = 0;   // all elements of the small tensor are visited; masked ones are stored as zeros
            M.dinner[w] = pl.prog.dinner[q];
            registers = registers && has_register_form(pl.prog.dinner[q]);
            blocks += (n + 63) / 64;
        }
        if (fits && M.count >= 2) {
            M.first[M.count] = (int32_t)blocks;
            TAD_LAUNCH_FORM(registers ? 1 : 0, "k_program_gather_multi", k_program_gather_multi, dim3((unsigned)blocks),
                            dim3(64), 0, s, M, n_ops, A, static_cast<const T *>(ws));
            return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
        }
    }
    // the gradient of a tensor is the sum over its occurrences: the first occurrence stores, aliases add
    for (size_t q = 0; q < pl.args.size(); ++q) {
        const size_t p = (size_t)pl.root[q];
        if (!dx[p]) continue;
        if (!pl.ap[q].derived) return TAD_EINVAL;
        const bool in_outer = (pl.prog.outer_mask >> q) & 1u;
        const bool inner_zero = pl.prog.dinner[q].result < 0;   // the inner function does not depend on this operand
        // a tensor one of whose occurrences is gathered over its unmasked elements only is cleared first, and
        // all its launches add
        bool cleared = false;
        for (size_t o = 0; o < pl.args.size(); ++o) {
            if ((size_t)pl.root[o] != p) continue;
            cleared = cleared || (pl.ap[o].derived && pl.ap[o].dev.live);
            cleared = cleared || (((pl.prog.outer_mask >> o) & 1u) && pl.ap_outer[o].derived && pl.ap_outer[o].dev.live);
        }
        if (cleared && q == p) {
            const long long count = pl.arg_count[p];
            TAD_LAUNCH("k_clear", (k_clear<T>), dim3(clear_blocks<T>(count)), dim3(256), 0, s,
                       static_cast<T *>(dx[p]), count);
            if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        }
        const int n = (int)gather_launch_count(pl.ap[q].dev, pl.arg_count[p]);   // element numbers of the launch
        const int form = program_form(has_register_form(pl.prog.dinner[q]), pl.terms_total / (double)(n > 0 ? n : 1));
        const GatherShape shape = gather_shape(pl.ap[q].dev, n, pl.terms_total);
        const int add_inner = (q != p || cleared) ? 1 : 0;
        if (in_outer && inner_zero) {
            // nothing to gather over the summation indices: the term of the outer function is the whole gradient
        } else if (shape.layout != kLayoutThreads) {
            const int splits = shape.splits;
            double *const partial = splits > 1 ? split_partial : nullptr;
            int32_t *const live = splits > 1 ? split_live(n, splits) : nullptr;
            if (shape.layout == kLayoutLanes)
                TAD_LAUNCH_FORM(form, "k_program_gather_lanes", k_program_gather_lanes, dim3((n + 255) / 256, splits),
                                dim3(256), 0, s, pl.ap[q].dev, pl.prog.dinner[q], (int)pl.args.size(), A,
                                static_cast<const T *>(ws), static_cast<T *>(dx[p]), n, add_inner, partial, live);
            else
                TAD_LAUNCH_FORM(form, "k_program_gather_coop", k_program_gather_coop, dim3(n, splits), dim3(256), 0, s,
                                pl.ap[q].dev, pl.prog.dinner[q], (int)pl.args.size(), A, static_cast<const T *>(ws),
                                static_cast<T *>(dx[p]), add_inner, partial, live);
            if (splits > 1) {
                if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
                TAD_LAUNCH("k_split_finish", (k_split_finish<T>), dim3((n + 3) / 4), dim3(256), 0, s,
                           (const double *)partial, (const int32_t *)live, splits, static_cast<T *>(dx[p]), n, add_inner);
            }
        } else {
            // workgroups of one wavefront, as for the generic kernels: a wavefront with a heavy element must not
            // hold the places of its finished neighbours
            TAD_LAUNCH_FORM(form, "k_program_gather", k_program_gather, dim3((n + 63) / 64), dim3(64), 0, s,
                            pl.ap[q].dev, pl.prog.dinner[q], (int)pl.args.size(), A, static_cast<const T *>(ws),
                            static_cast<T *>(dx[p]), n, add_inner, pl.terms_total >= (double)kHeavyTerms ? 1 : 0);
        }
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        if (!in_outer) continue;
        if (!pl.ap_outer[q].derived) return TAD_EINVAL;
        const int no = (int)gather_launch_count(pl.ap_outer[q].dev, pl.arg_count[p]);
        const int form_outer = program_form(has_register_form(pl.prog.douter_arg[q]), (double)pl.f_count / (double)(no > 0 ? no : 1));
        const int add_outer = (q != p || !inner_zero || cleared) ? 1 : 0;
        if (use_cooperative_gather(no, (double)pl.f_count)) {
            const int splits = cooperative_splits(no, (double)pl.f_count);
            double *const partial = splits > 1 ? split_partial : nullptr;
            int32_t *const live = splits > 1 ? split_live(no, splits) : nullptr;
            TAD_LAUNCH_FORM(form_outer, "k_program_gather_outer_coop", k_program_gather_outer_coop, dim3(no, splits),
                            dim3(256), 0, s, pl.ap_outer[q].dev, pl.prog.douter_arg[q], n_ops, pl.prog.outer_mask, A, s_ws,
                            static_cast<const T *>(df), static_cast<T *>(dx[p]), add_outer, partial, live);
            if (splits > 1) {
                if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
                TAD_LAUNCH("k_split_finish", (k_split_finish<T>), dim3((no + 3) / 4), dim3(256), 0, s,
                           (const double *)partial, (const int32_t *)live, splits, static_cast<T *>(dx[p]), no, add_outer);
            }
        } else {
            TAD_LAUNCH_FORM(form_outer, "k_program_gather_outer", k_program_gather_outer, dim3((no + 255) / 256),
                            dim3(256), 0, s, pl.ap_outer[q].dev, pl.prog.douter_arg[q], n_ops, pl.prog.outer_mask, A, s_ws,
                            static_cast<const T *>(df), static_cast<T *>(dx[p]), no, add_outer);
        }
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

int program_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                     hipStream_t s) {
    return pl.dtype == TAD_F64 ? bwd_t<double>(pl, args, df, dx, ws, s) : bwd_t<float>(pl, args, df, dx, ws, s);
}

}  // namespace tad
