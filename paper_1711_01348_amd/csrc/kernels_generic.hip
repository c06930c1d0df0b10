// Plan-driven generic kernels: the method exactly as stated.
//   forward: one thread per function index alpha, loop over the summation box (Sec. 5.1, 5.2)
//   gather:  one thread per gradient element beta: cokernel / divisibility / feasibility masks,
//            nested z loops with Fourier-Motzkin ranges, single store (final formula of Sec. 5.1)
// Works for every supported body and index matrix; the specialised families exist for speed only.
#include <hip/hip_runtime.h>

#include "bodies.h"
#include "gather_loop.h"
#include "launch.h"
#include "plan_dev.h"
#include "profile.h"

namespace tad {

// Sum of inner(values) over the summation box of function index `lin`, fp64.  `parts` cooperating threads share it:
// thread `part` takes the terms part, part + parts, ... of the box in row-major order (last summation index
// fastest), so that a wavefront reads neighbouring elements together.
template <int BODY, typename T>
__device__ __forceinline__ double forward_sum(const ForwardPlan &P, const ArgPtrs &A, int lin, int part, int parts) {
    constexpr int NA = BodyTraits<BODY>::NA;
    // The loops over the function indices are unrolled to the most indices a plan can have and cut short by tests
    // of the (uniform) rank: every field of the plan is then read from a fixed place in the kernel arguments, in one
    // go, instead of one dependent scalar load per turn of a loop (a thread without a sum spent most of its time
    // in those: 72 -> 50 us for f_ij = x_i^2 at 4096 x 4096).
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
    int64_t base[NA];
#pragma unroll
    for (int p = 0; p < NA; ++p) {
        int64_t o = P.base0[p];
#pragma unroll
        for (int d = 0; d < kMaxExt; ++d)
            if (d < P.n_f) o += P.off[p][d] * (int64_t)ext[d];
        base[p] = o;
    }
    int32_t k[kMaxExt] = {0};
    double acc = 0.0;
    const int last = P.n_sum - 1;
    const int32_t n_last = last >= 0 ? P.sum_n[last] : 1;
    if (P.n_cons == 0 && last >= 0 && (parts == 1 || last == 0 || n_last >= parts)) {
        // no extra conditions: the last summation index is a run of terms a constant stride apart; cooperating
        // threads take its terms in turn.  Whole batches of four terms are loaded before the first is used (one wait
        // for memory per batch, pointers advanced by additions, no predicates), the rest of the run goes one term at
        // a time; added in ascending order.  An operand that does not move along the run is loaded once per run.
        constexpr int U = 4;
        int64_t stp[NA];
        for (int p = 0; p < NA; ++p) stp[p] = P.last_stride[p] * parts;
        const int32_t mine = part < n_last ? (n_last - part + parts - 1) / parts : 0;
        for (;;) {
            const T *ptr[NA];
            T still[NA];
            for (int p = 0; p < NA; ++p) {
                int64_t o = base[p] + P.last_stride[p] * (int64_t)part;
                for (int sidx = 0; sidx < last; ++sidx) o += P.off[p][P.n_f + sidx] * (int64_t)k[sidx];
                ptr[p] = static_cast<const T *>(A.p[p]) + o;
                still[p] = stp[p] == 0 && mine > 0 ? *ptr[p] : T(0);
            }
            int32_t it = 0;
            for (; it + U <= mine; it += U) {
                T v[U][NA];
                for (int p = 0; p < NA; ++p) {
                    if (stp[p] == 0) {   // the same for the whole wavefront
#pragma unroll
                        for (int u = 0; u < U; ++u) v[u][p] = still[p];
                    } else {
                        const T *q = ptr[p];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            v[u][p] = *q;
                            q += stp[p];
                        }
                        ptr[p] = q;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) acc += (double)body_inner<BODY, T>(v[u]);
            }
            for (; it < mine; ++it) {
                T v[NA];
                for (int p = 0; p < NA; ++p) {
                    v[p] = stp[p] == 0 ? still[p] : *ptr[p];
                    ptr[p] += stp[p];
                }
                acc += (double)body_inner<BODY, T>(v);
            }
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
            T v[NA];
            for (int p = 0; p < NA; ++p) {
                int64_t o = base[p];
                for (int s = 0; s < P.n_sum; ++s) o += P.off[p][P.n_f + s] * (int64_t)k[s];
                v[p] = static_cast<const T *>(A.p[p])[o];
            }
            acc += (double)body_inner<BODY, T>(v);
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

template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_forward(const ForwardPlan P, const ArgPtrs A,
                                                         T *__restrict__ f, int nf) {
    const int lin = blockIdx.x * blockDim.x + threadIdx.x;
    if (lin >= nf) return;
    f[lin] = body_outer<BODY, T>((T)forward_sum<BODY, T>(P, A, lin, 0, 1));
}

// one block per function index (long sums)
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_forward_coop(const ForwardPlan P, const ArgPtrs A, T *__restrict__ f,
                                                              double *__restrict__ partial) {
    // gridDim.y blocks share a function index (few function indices): their sums go to `partial` and
    // k_generic_forward_finish applies the outer function
    __shared__ double red[4];
    const double total = block_sum_256(forward_sum<BODY, T>(P, A, blockIdx.x, (int)(blockIdx.y * 256 + threadIdx.x),
                                                            (int)(256 * gridDim.y)), red);
    if (threadIdx.x != 0) return;
    if (partial) partial[(size_t)blockIdx.x * gridDim.y + blockIdx.y] = total;
    else f[blockIdx.x] = body_outer<BODY, T>((T)total);
}

// one wavefront per function index: partial sums added in a fixed order, then the outer function
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_forward_finish(const double *__restrict__ partial, int splits,
                                                                T *__restrict__ f, int nf) {
    const int lin = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (lin >= nf) return;   // the whole wavefront leaves together
    double mine = 0.0;
    for (int sp = lane; sp < splits; sp += 64) mine += partial[(size_t)lin * splits + sp];
    const double total = wave_sum_all(mine);
    if (lane == 0) f[lin] = body_outer<BODY, T>((T)total);
}

// Element number `idx` of the launch over the gradient of operand p (gather_element_index: *lin receives its
// position in the tensor): masks, then the terms of the z loops shared by `parts` threads.
// Returns false (and *sum = 0) when a mask zeroes the element or the number is no element.
template <int BODY, typename T, int U = 4>
__device__ __forceinline__ bool gather_element(const GatherPlan &P, int p, const ArgPtrs &A, const T *__restrict__ f,
                                               const T *__restrict__ df, int idx, int *lin, int part, int parts,
                                               double *sum, int group = 0, int groups = 1) {
    constexpr int NA = BodyTraits<BODY>::NA;
    int32_t y[kMaxRank] = {0, 0, 0, 0};
    *sum = 0.0;
    if (!gather_element_index(P, idx, lin, y)) return false;
    double acc = 0.0;
    gather_loops(P, y, part, parts, [&](const int32_t *z, int32_t n, int32_t step) {
        // innermost run: offsets advance by a constant per term.  Whole batches of U terms are loaded before the
        // first of them is used, so that the loop waits for memory once per batch (U = 8 for the long runs of the
        // cooperative layouts: 4 and 16 measured slower); their offsets come from running 64-bit additions, no
        // multiplications and no predicates; what is left of the run goes one term at a time.  The terms are added
        // in ascending order.  An operand whose index does not move along the run (a_ik summed over j, ...) is
        // loaded once per run.
        int64_t off[NA + 1], stp[NA + 1];
        for (int q = 0; q < NA; ++q) {
            off[q] = gather_offset(P, q, y, z);
            stp[q] = P.offZ[q][0] * step;
        }
        off[NA] = gather_offset(P, kSlotF, y, z);
        stp[NA] = P.offZ[kSlotF][0] * step;
        T still[NA];
        for (int q = 0; q < NA; ++q) still[q] = stp[q] == 0 && n > 0 ? static_cast<const T *>(A.p[q])[off[q]] : T(0);
        int32_t it = 0;
        for (; it + U <= n; it += U) {
            T v[U][NA], fv[U], dfv[U];
            for (int q = 0; q < NA; ++q) {
                if (stp[q] == 0) {   // the same for the whole wavefront
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u][q] = still[q];
                } else {
                    int64_t o = off[q];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        v[u][q] = static_cast<const T *>(A.p[q])[o];
                        o += stp[q];
                    }
                    off[q] = o;
                }
            }
            {
                int64_t o = off[NA];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    fv[u] = f[o];
                    dfv[u] = df[o];
                    o += stp[NA];
                }
                off[NA] = o;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                acc += (double)(dfv[u] * body_douter<BODY, T>(fv[u], v[u]) * body_dinner<BODY, T>(p, v[u]));
        }
        for (; it < n; ++it) {
            T v[NA];
            for (int q = 0; q < NA; ++q) {
                v[q] = stp[q] == 0 ? still[q] : static_cast<const T *>(A.p[q])[off[q]];
                off[q] += stp[q];
            }
            const T fv = f[off[NA]], dfv = df[off[NA]];
            off[NA] += stp[NA];
            acc += (double)(dfv * body_douter<BODY, T>(fv, v) * body_dinner<BODY, T>(p, v));
        }
    }, group, groups);
    *sum = acc;
    return true;
}

// How many terms element number `idx` sums, roughly; 0 if it is masked out.
__device__ __forceinline__ int64_t element_estimate(const GatherPlan &P, int idx) {
    int32_t y[kMaxRank] = {0, 0, 0, 0};
    int lin;
    if (!gather_element_index(P, idx, &lin, y)) return 0;
    return gather_estimate(P, y);
}

// one thread per gradient element; an element with many terms (the masks can leave a few elements with all the
// work, e.g. the diagonal of a matrix that is read on its diagonal only) is summed by the whole wavefront
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_gather(const GatherPlan P, int p, const ArgPtrs A,
                                                        const T *__restrict__ f, const T *__restrict__ df,
                                                        T *__restrict__ dx, int n, int accumulate, int classify) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x, lane = threadIdx.x & 63;
    const bool inside = idx < n;
    // classify == 0: the whole expression has fewer terms than one heavy element would
    const bool heavy = classify && inside && element_estimate(P, idx) >= kHeavyTerms;
    double acc = 0.0;
    bool live = false;
    int lin = -1;
    if (inside && !heavy) live = gather_element<BODY, T>(P, p, A, f, df, idx, &lin, 0, 1, &acc);
    for (unsigned long long todo = __ballot(heavy); todo; todo &= todo - 1) {   // the same in every lane
        const int src = __ffsll((long long)todo) - 1;
        double part_sum;
        int lin_src;
        gather_element<BODY, T>(P, p, A, f, df, __shfl(idx, src, 64), &lin_src, lane, 64, &part_sum);
        const double total = wave_sum_all(part_sum);
        if (lane == src) { acc = total; live = true; lin = lin_src; }
    }
    if (!inside) return;
    // accumulate != 0: a further occurrence of the same tensor adds to what the earlier launches stored
    // (same owner thread, launches ordered on the stream: still no atomics)
    store_element(dx, lin, live, acc, accumulate);
}

// one block per gradient element (few elements, long sums): the 256 threads share the z loops and their partial
// sums are added in a fixed order
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_gather_coop(const GatherPlan P, int p, const ArgPtrs A,
                                                             const T *__restrict__ f, const T *__restrict__ df,
                                                             T *__restrict__ dx, int accumulate,
                                                             double *__restrict__ partial, int32_t *__restrict__ live_out) {
    // gridDim.y blocks share an element (partial != null then): block b takes the parts b * 256 ... of 256 gridDim.y
    __shared__ double red[4];
    // The accelerator dies take workgroups in turn, each with an L2 of its own.  Neighbouring elements often sum
    // over the same part of f (da_ik for k = 0 .. K-1: the same row; dd_m, dd_m+1: K-1 rows in common), so every
    // die gets a contiguous range of elements and neighbours run side by side on one die instead of fetching
    // that part once per die.
    int idx = blockIdx.x;
    if (gridDim.y == 1) {
        const int per_die = gridDim.x >> 3;
        if (idx < (per_die << 3)) idx = (idx & 7) * per_die + (idx >> 3);
    }
    double acc;
    int lin;
    const bool live = gather_element<BODY, T, 8>(P, p, A, f, df, idx, &lin, threadIdx.x, 256, &acc,
                                              (int)blockIdx.y, (int)gridDim.y);   // uniform over the block
    const double total = block_sum_256(acc, red);
    if (threadIdx.x != 0) return;
    if (partial) store_partial(partial, live_out, idx, lin, live, total);
    else store_element(dx, lin, live, total, accumulate);
}

// One wavefront per gradient element, four elements per workgroup: the form of the cooperative layout for gradients
// with many elements (thousands of long sums, e.g. da_ik, i < 8192: 8192 terms each).  With a whole workgroup per
// element a thread has only a few dozen terms, and walking the plan and adding up the workgroup cost as much as
// the terms; a wavefront has four times as many terms per lane and adds up with lane exchanges alone.
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_gather_wave(const GatherPlan P, int p, const ArgPtrs A,
                                                             const T *__restrict__ f, const T *__restrict__ df,
                                                             T *__restrict__ dx, int n, int accumulate) {
    // every die a contiguous range of workgroups (see k_generic_gather_coop)
    int blk = blockIdx.x;
    const int per_die = gridDim.x >> 3;
    if (blk < (per_die << 3)) blk = (blk & 7) * per_die + (blk >> 3);
    const int idx = blk * 4 + (int)(threadIdx.x >> 6);
    if (idx >= n) return;   // the whole wavefront leaves together
    double acc;
    int lin;
    const bool live = gather_element<BODY, T, 8>(P, p, A, f, df, idx, &lin, (int)(threadIdx.x & 63), 64, &acc);
    const double total = wave_sum_all(acc);
    if ((threadIdx.x & 63) == 0) store_element(dx, lin, live, total, accumulate);
}

// one thread per gradient element, the terms of every element shared by gridDim.y blocks (long sums read across
// the contiguous direction of f: neighbouring threads read neighbouring f)
template <int BODY, typename T>
__global__ __launch_bounds__(256) void k_generic_gather_lanes(const GatherPlan P, int p, const ArgPtrs A,
                                                              const T *__restrict__ f, const T *__restrict__ df,
                                                              T *__restrict__ dx, int n, int accumulate,
                                                              double *__restrict__ partial, int32_t *__restrict__ live_out) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    double acc;
    int lin;
    const bool live = gather_element<BODY, T, 8>(P, p, A, f, df, idx, &lin, 0, 1, &acc, (int)blockIdx.y, (int)gridDim.y);
    if (partial) store_partial(partial, live_out, idx, lin, live, acc);
    else store_element(dx, lin, live, acc, accumulate);
}

// Several gradients of small tensors in one launch: every kernel launch starts with cold instruction caches,
// and a wavefront that walks this code once spends most of its time fetching it (8 to 25 us per launch for a few
// dozen terms); in one launch the gradients pay that together instead of one after the other.  Workgroups of one
// wavefront; workgroup b works on gradient g with first[g] <= b < first[g + 1].
constexpr int kWaveElements = 4096;           // cooperative layout with at least this many elements: a wavefront each
constexpr long long kSpreadElements = 1024;   // up to this many gradient elements in all: a wavefront each
struct MultiGather {
    int32_t count;
    int32_t first[kMaxArgs + 1];
    int32_t n[kMaxArgs];         // elements of gradient g
    int32_t operand[kMaxArgs];   // operand whose plan and partial derivative gradient g uses
    void *dx[kMaxArgs];
    GatherPlan plan[kMaxArgs];
};
// SPREAD: for expressions with few gradient elements in all (the host checks): one workgroup, a single wavefront,
// per element; the lanes share its terms and add their sums in a fixed order, and none of the code for elements of
// very different weight is compiled in (700 instead of 5100 instructions for the worked expression in fp64).
// Such a launch waits for its instructions, not for its data: on the 8 x 6 x 5 worked expression a wavefront
// spends two thirds of its cycles waiting, 1.5 % of them for memory instructions (24.7 -> 22.2 us).
template <int BODY, typename T, bool SPREAD>
__global__ __launch_bounds__(64) void k_generic_gather_multi(const MultiGather M, const ArgPtrs A,
                                                             const T *__restrict__ f, const T *__restrict__ df,
                                                             int classify) {
    int g = 0;
    while (g + 1 < M.count && (int)blockIdx.x >= M.first[g + 1]) ++g;   // the same for the whole workgroup
    const int p = M.operand[g];
    if constexpr (SPREAD) {
        const GatherPlan &P = M.plan[g];
        double part_sum;
        int lin;
        const bool live = gather_element<BODY, T, 1>(P, p, A, f, df, (int)blockIdx.x - M.first[g], &lin, (int)threadIdx.x,
                                                     64, &part_sum);   // the same for all lanes
        const double total = wave_sum_all(part_sum);
        if (threadIdx.x == 0) store_element(static_cast<T *>(M.dx[g]), lin, live, total, 0);
        return;
    }
    const GatherPlan &P = M.plan[g];
    const int idx = ((int)blockIdx.x - M.first[g]) * 64 + (int)threadIdx.x, lane = threadIdx.x;
    const bool inside = idx < M.n[g];
    // as in k_generic_gather: an element with many terms is summed by the whole wavefront
    const bool heavy = classify && inside && element_estimate(P, idx) >= kHeavyTerms;
    double acc = 0.0;
    bool live = false;
    int lin = -1;
    if (inside && !heavy) live = gather_element<BODY, T>(P, p, A, f, df, idx, &lin, 0, 1, &acc);
    for (unsigned long long todo = __ballot(heavy); todo; todo &= todo - 1) {   // the same in every lane
        const int src = __ffsll((long long)todo) - 1;
        double part_sum;
        int lin_src;
        gather_element<BODY, T>(P, p, A, f, df, __shfl(idx, src, 64), &lin_src, lane, 64, &part_sum);
        const double total = wave_sum_all(part_sum);
        if (lane == src) { acc = total; live = true; lin = lin_src; }
    }
    if (!inside) return;
    store_element(static_cast<T *>(M.dx[g]), lin, live, acc, 0);
}

// Small expressions whose terms were listed at plan time: one workgroup, a single wavefront, per gradient element;
// lane l adds the terms l, l + 64, ... of the element's list and the lane sums are added in a fixed order.  An
// element without terms (masked out, or never referenced) is stored as zero.
struct ListedOut {
    void *dx[kMaxArgs];   // per gradient of the list; null: not wanted
};
template <int BODY, typename T>
__global__ __launch_bounds__(64) void k_generic_gather_listed(const TermList L, const ListedOut O, const ArgPtrs A,
                                                              const T *__restrict__ f, const T *__restrict__ df) {
    constexpr int NA = BodyTraits<BODY>::NA;
    const int e = blockIdx.x;
    int g = 0;
    while (g + 1 < L.n_grad && e >= L.first_element[g + 1]) ++g;   // the same for the whole workgroup
    T *const dx = static_cast<T *>(O.dx[g]);
    if (!dx) return;
    const int p = L.operand[g];
    double acc = 0.0;
    for (int t = L.first_term[e] + (int)threadIdx.x; t < (int)L.first_term[e + 1]; t += 64) {
        T v[NA];
        for (int q = 0; q < NA; ++q) v[q] = static_cast<const T *>(A.p[q])[L.off[t][q]];
        const int of = L.off[t][kListSlots - 1];
        acc += (double)(df[of] * body_douter<BODY, T>(f[of], v) * body_dinner<BODY, T>(p, v));
    }
    const double total = wave_sum_all(acc);
    if (threadIdx.x == 0) dx[e - L.first_element[g]] = (T)total;
}

template <int BODY, typename T>
static int launch_body(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                       void *const *dx, void *fout, void *ws, hipStream_t s) {
    ArgPtrs A{};
    for (size_t q = 0; q < pl.args.size(); ++q) A.p[q] = args[pl.root[q]];
    if (fout) {
        int nf = (int)pl.f_count;
        if (use_cooperative_gather(nf, pl.terms_total)) {   // every function index sums many terms
            const int splits = cooperative_splits(nf, pl.terms_total);
            if (splits > 1 && !ws) return TAD_ENOMEM;
            double *const partial = splits > 1 ? reinterpret_cast<double *>(static_cast<char *>(ws) + pl.split_ws_offset) : nullptr;
            TAD_LAUNCH("k_generic_forward_coop", (k_generic_forward_coop<BODY, T>), dim3(nf, splits), dim3(256), 0, s,
                       pl.fwd, A, static_cast<T *>(fout), partial);
            if (splits > 1) {
                if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
                TAD_LAUNCH("k_generic_forward_finish", (k_generic_forward_finish<BODY, T>), dim3((nf + 3) / 4), dim3(256),
                           0, s, (const double *)partial, splits, static_cast<T *>(fout), nf);
            }
        } else
            TAD_LAUNCH("k_generic_forward", (k_generic_forward<BODY, T>), dim3((nf + 255) / 256), dim3(256), 0, s, pl.fwd,
                       A, static_cast<T *>(fout), nf);
        return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
    }
    // a small expression with its terms listed at plan time: one launch for all its gradients
    if (!pl.term_list.empty()) {
        const TermList &L = pl.term_list[0];
        ListedOut O{};
        for (size_t q = 0; q < pl.args.size(); ++q)
            if (dx[q] && !pl.ap[q].derived) return TAD_EINVAL;
        bool any = false;
        for (int g = 0; g < L.n_grad; ++g) {
            O.dx[g] = dx[L.operand[g]];
            any = any || O.dx[g];
        }
        if (!any) return TAD_OK;
        TAD_LAUNCH("k_generic_gather_listed", (k_generic_gather_listed<BODY, T>), dim3((unsigned)L.first_element[L.n_grad]),
                   dim3(64), 0, s, L, O, A, static_cast<const T *>(f), static_cast<const T *>(df));
        return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
    }
    // an expression without aliases whose gradients are all small tensors with short sums: one launch for all
    if (!pl.has_alias) {
        MultiGather M{};
        bool fits = true;
        long long blocks = 0, elements = 0;
        for (size_t q = 0; q < pl.args.size() && fits; ++q) {
            if (!dx[q]) continue;
            const long long n = pl.arg_count[q];
            fits = pl.ap[q].family == TAD_FAMILY_GENERIC && pl.ap[q].derived && n <= (1 << 16) &&
                   gather_shape(pl.ap[q].dev, n, pl.terms_total).layout == kLayoutThreads;
            if (!fits) break;
            const int g = M.count++;
            M.first[g] = (int32_t)blocks;
            M.n[g] = (int32_t)n;
            M.operand[g] = (int32_t)q;
            M.dx[g] = dx[q];
            M.plan[g] = pl.ap[q].dev;
            M.plan[g].live = 0;   // all elements of the small tensor are visited; masked ones are stored as zeros
            blocks += (n + 63) / 64;
            elements += n;
        }
        if (fits && M.count >= 2) {
            M.first[M.count] = (int32_t)blocks;
            if (elements <= kSpreadElements) {
                // one wavefront per element: the first workgroup of gradient g is the sum of the earlier gradients' elements
                long long first = 0;
                for (int g = 0; g < M.count; ++g) {
                    M.first[g] = (int32_t)first;
                    first += M.n[g];
                }
                M.first[M.count] = (int32_t)first;
                TAD_LAUNCH("k_generic_gather_multi", (k_generic_gather_multi<BODY, T, true>), dim3((unsigned)first), dim3(64),
                           0, s, M, A, static_cast<const T *>(f), static_cast<const T *>(df), 0);
            } else
                TAD_LAUNCH("k_generic_gather_multi", (k_generic_gather_multi<BODY, T, false>), dim3((unsigned)blocks), dim3(64),
                           0, s, M, A, static_cast<const T *>(f), static_cast<const T *>(df),
                           pl.terms_total >= (double)kHeavyTerms ? 1 : 0);
            return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
        }
    }
    // the gradient of a tensor is the sum over its occurrences (Sec. 5.3): the first occurrence stores,
    // every alias operand adds in a launch of its own
    for (size_t q = 0; q < pl.args.size(); ++q) {
        const size_t p = (size_t)pl.root[q];
        if (!dx[p] || pl.ap[q].family != TAD_FAMILY_GENERIC) continue;
        if (!pl.ap[q].derived) return TAD_EINVAL;
        // a tensor one of whose occurrences is gathered over its unmasked elements only is cleared first, and
        // all its launches add
        bool cleared = false;
        for (size_t o = 0; o < pl.args.size(); ++o) cleared = cleared || ((size_t)pl.root[o] == p && pl.ap[o].derived && pl.ap[o].dev.live);
        if (cleared && q == p) {
            const long long count = pl.arg_count[p];
            TAD_LAUNCH("k_clear", (k_clear<T>), dim3(clear_blocks<T>(count)), dim3(256), 0, s,
                       static_cast<T *>(dx[p]), count);
            if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        }
        const int accumulate = (q != p || cleared) ? 1 : 0;
        const int n = (int)gather_launch_count(pl.ap[q].dev, pl.arg_count[p]);   // element numbers of the launch
        const GatherShape shape = gather_shape(pl.ap[q].dev, n, pl.terms_total);
        if (shape.layout != kLayoutThreads) {
            const int splits = shape.splits;
            double *partial = nullptr;
            int32_t *live = nullptr;
            if (splits > 1) {
                if (!ws) return TAD_ENOMEM;
                partial = reinterpret_cast<double *>(static_cast<char *>(ws) + pl.split_ws_offset);
                live = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(partial) + align256((size_t)n * splits * 8));
            }
            if (shape.layout == kLayoutLanes)
                TAD_LAUNCH("k_generic_gather_lanes", (k_generic_gather_lanes<BODY, T>), dim3((n + 255) / 256, splits),
                           dim3(256), 0, s, pl.ap[q].dev, (int)q, A, static_cast<const T *>(f), static_cast<const T *>(df),
                           static_cast<T *>(dx[p]), n, accumulate, partial, live);
            else if (splits == 1 && n >= kWaveElements)
                TAD_LAUNCH("k_generic_gather_wave", (k_generic_gather_wave<BODY, T>), dim3((n + 3) / 4), dim3(256), 0, s,
                           pl.ap[q].dev, (int)q, A, static_cast<const T *>(f), static_cast<const T *>(df),
                           static_cast<T *>(dx[p]), n, accumulate);
            else
                TAD_LAUNCH("k_generic_gather_coop", (k_generic_gather_coop<BODY, T>), dim3(n, splits), dim3(256), 0, s,
                           pl.ap[q].dev, (int)q, A, static_cast<const T *>(f), static_cast<const T *>(df),
                           static_cast<T *>(dx[p]), accumulate, partial, live);
            if (splits > 1) {
                if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
                TAD_LAUNCH("k_split_finish", (k_split_finish<T>), dim3((n + 3) / 4), dim3(256), 0, s,
                           (const double *)partial, (const int32_t *)live, splits, static_cast<T *>(dx[p]), n, accumulate);
            }
        } else
            // workgroups of one wavefront: a wavefront that sums a heavy element runs long after its neighbours
            // have left, and in a larger workgroup it would keep their places taken (2.8 -> 1.1 ms for dc of the
            // worked expression at 8192 x 8192: 67 million elements, 8192 of them heavy)
            TAD_LAUNCH("k_generic_gather", (k_generic_gather<BODY, T>), dim3((n + 63) / 64), dim3(64), 0, s,
                       pl.ap[q].dev, (int)q, A, static_cast<const T *>(f), static_cast<const T *>(df),
                       static_cast<T *>(dx[p]), n, accumulate, pl.terms_total >= (double)kHeavyTerms ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

template <typename T>
static int launch_dtype(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                        void *const *dx, void *fout, void *ws, hipStream_t s) {
    switch (pl.expr.body) {
    case TAD_BODY_SQ: return launch_body<TAD_BODY_SQ, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_CUBE: return launch_body<TAD_BODY_CUBE, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_SIN: return launch_body<TAD_BODY_SIN, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_EXP: return launch_body<TAD_BODY_EXP, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_MUL: return launch_body<TAD_BODY_MUL, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_WORKED: return launch_body<TAD_BODY_WORKED, T>(pl, args, f, df, dx, fout, ws, s);
    case TAD_BODY_TANH_DOT: return launch_body<TAD_BODY_TANH_DOT, T>(pl, args, f, df, dx, fout, ws, s);
    default: return TAD_EUNSUPPORTED;
    }
}

int generic_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s) {
    return pl.dtype == TAD_F64 ? launch_dtype<double>(pl, args, nullptr, nullptr, nullptr, f, ws, s)
                               : launch_dtype<float>(pl, args, nullptr, nullptr, nullptr, f, ws, s);
}

// Launches the generic gather kernel for every wanted gradient whose family is GENERIC.
int generic_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                     void *const *dx, void *ws, hipStream_t s) {
    return pl.dtype == TAD_F64 ? launch_dtype<double>(pl, args, f, df, dx, nullptr, ws, s)
                               : launch_dtype<float>(pl, args, f, df, dx, nullptr, ws, s);
}

}  // namespace tad
