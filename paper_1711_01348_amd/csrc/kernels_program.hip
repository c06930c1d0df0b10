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
#include "worked_geom.h"

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

// One pass over the operations; temporaries live in the thread's private memory.
template <typename T>
__device__ T prog_eval(const DevProg &P, const T *v, T s) {
    if (P.result < 0) return T(0);
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
        case P_NEG: r = -t[a]; break;
        case P_EXP: r = Fn<T>::exp_(t[a]); break;
        case P_LOG: r = Fn<T>::log_(t[a]); break;
        case P_SIN: r = Fn<T>::sin_(t[a]); break;
        case P_COS: r = Fn<T>::cos_(t[a]); break;
        case P_TANH: r = Fn<T>::tanh_(t[a]); break;
        case P_SQRT: r = Fn<T>::sqrt_(t[a]); break;
        case P_POWI: {
            const T x = t[a];
            r = x;
            for (int e = 1; e < P.k[i]; ++e) r *= x;
            break;
        }
        default: r = T(0);
        }
        t[i] = r;
    }
    return t[P.result];
}

// sum over the summation box of inner(values) for one function index, fp64 accumulation; base[p] receives the
// offset of operand p at the first summation index (for an operand that ignores the summation indices: its
// offset at this function index)
// `parts` cooperating threads share the sum: thread `part` takes the terms part, part + parts, ... of the box
// in row-major order (last summation index fastest), so that a wavefront reads neighbouring elements together.
template <typename T>
__device__ double inner_sum(const ForwardPlan &P, const DevProg &inner, int n_ops, const ArgPtrs &A, int lin,
                            int64_t *base, int part = 0, int parts = 1) {
    int32_t ext[kMaxExt];
    {
        int t = lin;
        for (int d = P.n_f - 1; d >= 0; --d) { ext[d] = t % P.f_shape[d]; t /= P.f_shape[d]; }
    }
    for (int p = 0; p < n_ops; ++p) {
        int64_t o = 0;
        for (int d = 0; d < P.n_f; ++d) o += P.off[p][d] * (int64_t)ext[d];
        for (int s = 0; s < P.n_sum; ++s) o += P.off[p][P.n_f + s] * (int64_t)P.sum_lo[s];
        base[p] = o;
    }
    int32_t k[kMaxExt] = {0};
    double acc = 0.0;
    auto term = [&]() {
        if (forward_conditions(P, ext, k)) {   // a term outside the extra conditions is not part of the sum
            T v[kMaxArgs];
            for (int p = 0; p < n_ops; ++p) {
                int64_t o = base[p];
                for (int s = 0; s < P.n_sum; ++s) o += P.off[p][P.n_f + s] * (int64_t)k[s];
                v[p] = static_cast<const T *>(A.p[p])[o];
            }
            acc += (double)prog_eval<T>(inner, v, T(0));
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
template <typename T>
__global__ __launch_bounds__(256) void k_program_forward(const ForwardPlan P, const DevProg inner, const DevProg outer,
                                                         int n_ops, uint32_t outer_mask, const ArgPtrs A,
                                                         const T *__restrict__ df, T *__restrict__ out,
                                                         T *__restrict__ s_out, int nf) {
    const int lin = blockIdx.x * blockDim.x + threadIdx.x;
    if (lin >= nf) return;
    int64_t base[kMaxArgs];
    const T s = (T)inner_sum<T>(P, inner, n_ops, A, lin, base);
    T v[kMaxArgs];
    for (int p = 0; p < n_ops; ++p) v[p] = ((outer_mask >> p) & 1u) ? static_cast<const T *>(A.p[p])[base[p]] : T(0);
    const T o = prog_eval<T>(outer, v, s);
    out[lin] = df ? df[lin] * o : o;
    if (s_out) s_out[lin] = s;
}

// the same with one block per function index (long sums): the 256 threads share the sum
template <typename T>
__global__ __launch_bounds__(256) void k_program_forward_coop(const ForwardPlan P, const DevProg inner, const DevProg outer,
                                                              int n_ops, uint32_t outer_mask, const ArgPtrs A,
                                                              const T *__restrict__ df, T *__restrict__ out,
                                                              T *__restrict__ s_out) {
    __shared__ double red[4];
    const int lin = blockIdx.x;
    int64_t base[kMaxArgs];
    const double mine = inner_sum<T>(P, inner, n_ops, A, lin, base, threadIdx.x, 256);
    const T s = (T)block_sum_256(mine, red);
    if (threadIdx.x != 0) return;
    T v[kMaxArgs];
    for (int p = 0; p < n_ops; ++p) v[p] = ((outer_mask >> p) & 1u) ? static_cast<const T *>(A.p[p])[base[p]] : T(0);
    const T o = prog_eval<T>(outer, v, s);
    out[lin] = df ? df[lin] * o : o;
    if (s_out) s_out[lin] = s;
}

// Term df * d outer / d x^p of gradient element `lin` of an operand the outer function reads: masks and ranges from
// the operand's plan over the function indices alone.
template <typename T>
__device__ __forceinline__ bool outer_element(const GatherPlan &P, const DevProg &douter_p, int n_ops, uint32_t outer_mask,
                                              const ArgPtrs &A, const T *__restrict__ s_ws, const T *__restrict__ df,
                                              int lin, int part, int parts, double *sum) {
    int32_t beta[kMaxRank], y[kMaxRank] = {0, 0, 0, 0};
    {
        int t = lin;
        for (int r = P.rank - 1; r >= 0; --r) { beta[r] = t % P.shape[r]; t /= P.shape[r]; }
    }
    *sum = 0.0;
    if (!gather_prepare(P, beta, y)) return false;
    double acc = 0.0;
    gather_loops(P, y, part, parts, [&](const int32_t *z, int32_t n, int32_t step) {
        int64_t off[kMaxArgs + 1];
        for (int q = 0; q < n_ops; ++q) off[q] = ((outer_mask >> q) & 1u) ? gather_offset(P, q, y, z) : 0;
        off[kMaxArgs] = gather_offset(P, kSlotF, y, z);
        for (int32_t it = 0; it < n; ++it) {
            T v[kMaxArgs];
            for (int q = 0; q < n_ops; ++q) v[q] = ((outer_mask >> q) & 1u) ? static_cast<const T *>(A.p[q])[off[q]] : T(0);
            acc += (double)(df[off[kMaxArgs]] * prog_eval<T>(douter_p, v, s_ws[off[kMaxArgs]]));
            for (int q = 0; q < n_ops; ++q) off[q] += ((outer_mask >> q) & 1u) ? P.offZ[q][0] * step : 0;
            off[kMaxArgs] += P.offZ[kSlotF][0] * step;
        }
    });
    *sum = acc;
    return true;
}

template <typename T>
__global__ __launch_bounds__(256) void k_program_gather_outer(const GatherPlan P, const DevProg douter_p, int n_ops,
                                                              uint32_t outer_mask, const ArgPtrs A,
                                                              const T *__restrict__ s_ws, const T *__restrict__ df,
                                                              T *__restrict__ dx, int n, int accumulate) {
    const int lin = blockIdx.x * blockDim.x + threadIdx.x;
    if (lin >= n) return;
    double acc;
    if (!outer_element<T>(P, douter_p, n_ops, outer_mask, A, s_ws, df, lin, 0, 1, &acc)) {
        if (!accumulate) dx[lin] = T(0);
        return;
    }
    dx[lin] = (accumulate ? dx[lin] : T(0)) + (T)acc;
}

// one block per gradient element (few elements, many function indices each)
template <typename T>
__global__ __launch_bounds__(256) void k_program_gather_outer_coop(const GatherPlan P, const DevProg douter_p, int n_ops,
                                                                   uint32_t outer_mask, const ArgPtrs A,
                                                                   const T *__restrict__ s_ws, const T *__restrict__ df,
                                                                   T *__restrict__ dx, int accumulate) {
    __shared__ double red[4];
    const int lin = blockIdx.x;
    double acc;
    const bool live = outer_element<T>(P, douter_p, n_ops, outer_mask, A, s_ws, df, lin, threadIdx.x, 256, &acc);
    const double total = block_sum_256(acc, red);
    if (threadIdx.x != 0) return;
    if (!live) {
        if (!accumulate) dx[lin] = T(0);
        return;
    }
    dx[lin] = (accumulate ? dx[lin] : T(0)) + (T)total;
}

// Gradient element `lin`: masks, then the terms of the z loops shared by `parts` threads.
template <typename T>
__device__ __forceinline__ bool program_element(const GatherPlan &P, const DevProg &dinner, int n_ops, const ArgPtrs &A,
                                                const T *__restrict__ g, int lin, int part, int parts, double *sum) {
    int32_t beta[kMaxRank], y[kMaxRank] = {0, 0, 0, 0};
    {
        int t = lin;
        for (int r = P.rank - 1; r >= 0; --r) { beta[r] = t % P.shape[r]; t /= P.shape[r]; }
    }
    *sum = 0.0;
    if (!gather_prepare(P, beta, y)) return false;
    double acc = 0.0;
    gather_loops(P, y, part, parts, [&](const int32_t *z, int32_t n, int32_t step) {
        int64_t off[kMaxArgs + 1];
        for (int q = 0; q < n_ops; ++q) off[q] = gather_offset(P, q, y, z);
        off[kMaxArgs] = gather_offset(P, kSlotF, y, z);
        for (int32_t it = 0; it < n; ++it) {
            T v[kMaxArgs];
            for (int q = 0; q < n_ops; ++q) v[q] = static_cast<const T *>(A.p[q])[off[q]];
            acc += (double)(g[off[kMaxArgs]] * prog_eval<T>(dinner, v, T(0)));
            for (int q = 0; q < n_ops; ++q) off[q] += P.offZ[q][0] * step;
            off[kMaxArgs] += P.offZ[kSlotF][0] * step;
        }
    });
    *sum = acc;
    return true;
}

template <typename T>
__global__ __launch_bounds__(256) void k_program_gather(const GatherPlan P, const DevProg dinner, int n_ops,
                                                        const ArgPtrs A, const T *__restrict__ g,
                                                        T *__restrict__ dx, int n, int accumulate, int classify) {
    const int lin = blockIdx.x * blockDim.x + threadIdx.x, lane = threadIdx.x & 63;
    const bool inside = lin < n;
    bool heavy = false;
    if (classify && inside) {   // classify == 0: the whole expression has fewer terms than one heavy element would
        int32_t beta[kMaxRank], y[kMaxRank] = {0, 0, 0, 0};
        int t = lin;
        for (int r = P.rank - 1; r >= 0; --r) { beta[r] = t % P.shape[r]; t /= P.shape[r]; }
        heavy = gather_prepare(P, beta, y) && gather_estimate(P, y) >= kHeavyTerms;
    }
    double acc = 0.0;
    bool live = false;
    if (inside && !heavy) live = program_element<T>(P, dinner, n_ops, A, g, lin, 0, 1, &acc);
    // an element with many terms is summed by the whole wavefront (the masks can leave few elements with all the work)
    for (unsigned long long todo = __ballot(heavy); todo; todo &= todo - 1) {
        const int src = __ffsll((long long)todo) - 1;
        double part_sum;
        program_element<T>(P, dinner, n_ops, A, g, __shfl(lin, src, 64), lane, 64, &part_sum);
        const double total = wave_sum_all(part_sum);
        if (lane == src) { acc = total; live = true; }
    }
    if (!inside) return;
    if (!live) {
        if (!accumulate) dx[lin] = T(0);
        return;
    }
    dx[lin] = (accumulate ? dx[lin] : T(0)) + (T)acc;
}

// one block per gradient element (few elements, long sums)
template <typename T>
__global__ __launch_bounds__(256) void k_program_gather_coop(const GatherPlan P, const DevProg dinner, int n_ops,
                                                             const ArgPtrs A, const T *__restrict__ g,
                                                             T *__restrict__ dx, int accumulate) {
    __shared__ double red[4];
    const int lin = blockIdx.x;
    double acc;
    const bool live = program_element<T>(P, dinner, n_ops, A, g, lin, threadIdx.x, 256, &acc);
    const double total = block_sum_256(acc, red);
    if (threadIdx.x != 0) return;
    if (!live) {
        if (!accumulate) dx[lin] = T(0);
        return;
    }
    dx[lin] = (accumulate ? dx[lin] : T(0)) + (T)total;
}

template <typename T>
static int fwd_t(const tad_plan &pl, const void *const *args, const void *df, void *out, void *s_out, hipStream_t s) {
    ArgPtrs A{};
    for (size_t q = 0; q < pl.args.size(); ++q) A.p[q] = args[pl.root[q]];
    const int nf = (int)pl.f_count;
    if (use_cooperative_gather(nf, pl.terms_total))   // every function index sums many terms
        TAD_LAUNCH("k_program_forward_coop", (k_program_forward_coop<T>), dim3(nf), dim3(256), 0, s, pl.fwd,
                   pl.prog.inner, df ? pl.prog.douter : pl.prog.outer, (int)pl.args.size(), pl.prog.outer_mask, A,
                   static_cast<const T *>(df), static_cast<T *>(out), static_cast<T *>(s_out));
    else
        TAD_LAUNCH("k_program_forward", (k_program_forward<T>), dim3((nf + 255) / 256), dim3(256), 0, s, pl.fwd,
                   pl.prog.inner, df ? pl.prog.douter : pl.prog.outer, (int)pl.args.size(), pl.prog.outer_mask, A,
                   static_cast<const T *>(df), static_cast<T *>(out), static_cast<T *>(s_out), nf);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

int program_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s) {
    return pl.dtype == TAD_F64 ? fwd_t<double>(pl, args, nullptr, f, nullptr, s)
                               : fwd_t<float>(pl, args, nullptr, f, nullptr, s);
}

template <typename T>
static int bwd_t(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                 hipStream_t s) {
    // workspace: g = df * (d outer / d sum), then (only if the outer function reads operands) the sums themselves
    T *const s_ws = pl.prog.outer_mask
                        ? reinterpret_cast<T *>(static_cast<char *>(ws) + align256((size_t)pl.f_count * sizeof(T)))
                        : nullptr;
    int rc = fwd_t<T>(pl, args, df, ws, s_ws, s);
    if (rc) return rc;
    ArgPtrs A{};
    for (size_t q = 0; q < pl.args.size(); ++q) A.p[q] = args[pl.root[q]];
    const int n_ops = (int)pl.args.size();
    // the gradient of a tensor is the sum over its occurrences: the first occurrence stores, aliases add
    for (size_t q = 0; q < pl.args.size(); ++q) {
        const size_t p = (size_t)pl.root[q];
        if (!dx[p]) continue;
        if (!pl.ap[q].derived) return TAD_EINVAL;
        const int n = (int)pl.arg_count[p];
        const bool in_outer = (pl.prog.outer_mask >> q) & 1u;
        const bool inner_zero = pl.prog.dinner[q].result < 0;   // the inner function does not depend on this operand
        if (in_outer && inner_zero) {
            // nothing to gather over the summation indices: the term of the outer function is the whole gradient
        } else if (use_cooperative_gather(n, pl.terms_total))
            TAD_LAUNCH("k_program_gather_coop", (k_program_gather_coop<T>), dim3(n), dim3(256), 0, s, pl.ap[q].dev,
                       pl.prog.dinner[q], (int)pl.args.size(), A, static_cast<const T *>(ws), static_cast<T *>(dx[p]),
                       q != p ? 1 : 0);
        else
            TAD_LAUNCH("k_program_gather", (k_program_gather<T>), dim3((n + 255) / 256), dim3(256), 0, s, pl.ap[q].dev,
                       pl.prog.dinner[q], (int)pl.args.size(), A, static_cast<const T *>(ws), static_cast<T *>(dx[p]), n,
                       q != p ? 1 : 0, pl.terms_total >= (double)kHeavyTerms ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        if (!in_outer) continue;
        if (!pl.ap_outer[q].derived) return TAD_EINVAL;
        const int accumulate = (q != p || !inner_zero) ? 1 : 0;
        if (use_cooperative_gather(n, (double)pl.f_count))
            TAD_LAUNCH("k_program_gather_outer_coop", (k_program_gather_outer_coop<T>), dim3(n), dim3(256), 0, s,
                       pl.ap_outer[q].dev, pl.prog.douter_arg[q], n_ops, pl.prog.outer_mask, A, s_ws,
                       static_cast<const T *>(df), static_cast<T *>(dx[p]), accumulate);
        else
            TAD_LAUNCH("k_program_gather_outer", (k_program_gather_outer<T>), dim3((n + 255) / 256), dim3(256), 0, s,
                       pl.ap_outer[q].dev, pl.prog.douter_arg[q], n_ops, pl.prog.outer_mask, A, s_ws,
                       static_cast<const T *>(df), static_cast<T *>(dx[p]), n, accumulate);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

int program_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                     hipStream_t s) {
    return pl.dtype == TAD_F64 ? bwd_t<double>(pl, args, df, dx, ws, s) : bwd_t<float>(pl, args, df, dx, ws, s);
}

}  // namespace tad
