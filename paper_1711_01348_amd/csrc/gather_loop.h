// Nested loops over the kernel coordinates z of one gradient element (final formula of Sec. 5.1): ranges from the
// plan's Fourier-Motzkin rows, outermost coordinate z_{kappa-1} first.  The loops can be shared by `parts`
// cooperating threads (all of them call with the same element), and by `groups` groups of such threads (blocks):
//   one group
//   - one coordinate: the threads take its values in turn (thread `part` takes every parts-th value, so that the
//     threads of a wavefront read neighbouring elements together);
//   - several, and the outermost has at least parts / 8 values: thread `part` takes every parts-th of them;
//   - otherwise every thread walks the outer coordinates, the values of an innermost run of at least `parts`
//     values are taken in turn, and shorter runs are dealt out whole to the threads in turn (a short outer range
//     over long inner runs would leave most threads idle the other way).
//   several groups
//   - one coordinate: all threads of all groups take its values in turn;
//   - two: the groups take the values of the outer one in turn, the threads of a group those of every run;
//   - more: the groups take the values of the outermost coordinate in turn, the threads of a group those of the
//     next one (every thread then evaluates only the ranges of the runs it sums itself: with many threads
//     walking all ranges costs more than the terms).
// `run(z, count, step)` is called once per innermost run with z[0] at the caller's first value; it handles the
// `count` values z[0], z[0] + step, ... itself (offsets advance by a constant per value there).
#pragma once
#include <hip/hip_runtime.h>

#include "plan_dev.h"
#include "launch_geom.h"

namespace tad {

template <class Run>
__device__ __forceinline__ void gather_loops(const GatherPlan &P, const int32_t *y, int part, int parts, Run &&run,
                                             int group = 0, int groups = 1) {
    // `run` is expanded in line: the walk below is arranged so that it is called from one place only
    int32_t z[kMaxKernel] = {0, 0, 0, 0}, hi[kMaxKernel] = {0, 0, 0, 0};
    // first value (relative to the range's start) and step of the outermost coordinate and of the one below it;
    // plain variables: arrays indexed by the level would be placed in LDS
    int32_t first_top = 0, step_top = 1, first_sub = 0, step_sub = 1;
    int sub = -1;   // the coordinate below the outermost one if the threads take its values in turn
    const int top = P.kappa - 1;
    bool single = false;         // exactly one run: no coordinate at all, or one coordinate shared by the threads
    bool share_runs = false;     // long runs taken in turn, short ones dealt out whole
    bool strided_runs = false;   // every run taken in turn
    int32_t count = 1, step = 1;
    if (P.kappa == 0) {
        if (part != 0 || group != 0) return;   // a single term: z is empty
        single = true;
    } else {
        gather_bounds(P, top, y, z, z[top], hi[top]);
        if (top == 0) {
            part += group * parts;
            parts *= groups;
            if (parts > 1) {
                const int64_t first = (int64_t)z[0] + part;
                if (first > hi[0]) return;
                z[0] = (int32_t)first;
                count = (int32_t)((hi[0] - first) / parts + 1);
                step = parts;
                single = true;
            }
        } else if (groups > 1) {
            first_top = group;
            step_top = groups;
            if (top == 1) {
                strided_runs = parts > 1;
            } else {
                sub = top - 1;
                first_sub = part;
                step_sub = parts;
            }
        } else if (parts > 1) {
            if (((int64_t)hi[top] - z[top] + 1) * 8 >= parts) {
                first_top = part;
                step_top = parts;
            } else {
                share_runs = true;
            }
        }
        if (top > 0) z[top] += first_top;   // may pass hi[top]: the walk ends at once
    }
    int turn = 0;   // whose turn it is to take a short run
    int lvl = top;
    for (;;) {
        bool mine = true;
        if (!single) {
            // walk to the next innermost run
            for (;;) {
                if (z[lvl] > hi[lvl]) {
                    if (++lvl > top) return;
                    z[lvl] += lvl == top ? step_top : lvl == sub ? step_sub : 1;
                } else if (lvl == 0) {
                    break;
                } else {
                    --lvl;
                    gather_bounds(P, lvl, y, z, z[lvl], hi[lvl]);
                    if (lvl == sub) z[lvl] += first_sub;
                }
            }
            count = hi[0] - z[0] + 1;   // >= 1 here
            step = 1;
            if (strided_runs || (share_runs && count >= parts)) {
                z[0] += part;
                mine = z[0] <= hi[0];
                count = mine ? (hi[0] - z[0]) / parts + 1 : 0;
                step = parts;
            } else if (share_runs) {
                mine = turn == part;
                turn = turn + 1 == parts ? 0 : turn + 1;
            }
        }
        if (mine) run(z, count, step);
        if (single) return;
        z[0] = hi[0] + 1;
    }
}

// Rough number of terms of one element: the lengths of the ranges multiplied, every range taken with the outer
// coordinates at their first values (exact when the ranges do not depend on each other).
__device__ __forceinline__ int64_t gather_estimate(const GatherPlan &P, const int32_t *y) {
    int32_t z[kMaxKernel] = {0, 0, 0, 0};
    int64_t n = 1;
    for (int lvl = P.kappa - 1; lvl >= 0; --lvl) {
        int32_t lo, hi;
        gather_bounds(P, lvl, y, z, lo, hi);
        if (hi < lo) return 0;
        n *= (int64_t)hi - lo + 1;
        z[lvl] = lo;
    }
    return n;
}

// An element with at least this many terms is summed by its whole wavefront instead of its own thread.
constexpr int64_t kHeavyTerms = 512;

// Sum over the 64 lanes, fixed order, result in every lane.
__device__ __forceinline__ double wave_sum_all(double v) {
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Sum of one double per thread over the block (256 threads), fixed order; the total is returned to thread 0.
__device__ __forceinline__ double block_sum_256(double v, double *red /* [4] in LDS */) {
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// Result of element number idx at position lin (lin < 0: no element): masked elements are stored as zeros unless
// the launch adds to what is there or runs over the unmasked elements only (the tensor was cleared before).
template <typename T>
__device__ __forceinline__ void store_element(T *__restrict__ dx, int lin, bool live, double total, int accumulate) {
    if (lin < 0) return;
    if (!live) {
        if (!accumulate) dx[lin] = T(0);
        return;
    }
    dx[lin] = (accumulate ? dx[lin] : T(0)) + (T)total;
}
// The same into the partial sums of an element shared by several workgroups: flag = position, -1 masked (store a
// zero at idx), -2 nothing to store.
__device__ __forceinline__ void store_partial(double *__restrict__ partial, int32_t *__restrict__ flag, int idx,
                                              int lin, bool live, double total) {
    partial[(size_t)idx * gridDim.y + blockIdx.y] = live ? total : 0.0;
    if (blockIdx.y == 0) flag[idx] = live ? lin : lin >= 0 ? -1 : -2;
}

// Finishing pass of a gradient whose elements were shared by several blocks: one wavefront per element, lane l
// adds the partial sums l, l + 64, ... in ascending order and the 64 lane sums are added in a fixed tree (a
// single thread would wait for one load after the other).  flag: see store_partial.
template <typename T>
__global__ __launch_bounds__(256) void k_split_finish(const double *__restrict__ partial, const int32_t *__restrict__ flag,
                                                      int splits, T *__restrict__ dx, int n, int accumulate) {
    const int idx = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (idx >= n) return;   // the whole wavefront leaves together
    double mine = 0.0;
    for (int sp = lane; sp < splits; sp += 64) mine += partial[(size_t)idx * splits + sp];
    const double total = wave_sum_all(mine);
    if (lane != 0) return;
    const int32_t where = flag[idx];
    store_element(dx, where >= 0 ? where : where == -1 ? idx : -1, where >= 0, total, accumulate);
}

// Clears a gradient before a launch that visits its unmasked elements only (a kernel rather than a memset, so
// that the call can be recorded into a graph).
template <typename T>
__global__ __launch_bounds__(256) void k_clear(T *__restrict__ dx, long long n) {
    // 16 bytes per thread where the tensor starts on a 16-byte boundary (it does when it is an allocation of its own)
    constexpr int V = 16 / (int)sizeof(T);
    typedef T vec __attribute__((ext_vector_type(V)));
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= n) return;
    if ((reinterpret_cast<uintptr_t>(dx) & 15) == 0 && i + V <= n) {
        vec zero;
        for (int v = 0; v < V; ++v) zero[v] = T(0);
        __builtin_nontemporal_store(zero, reinterpret_cast<vec *>(dx + i));
    } else {
        for (int v = 0; v < V && i + v < n; ++v) dx[i + v] = T(0);
    }
}
// number of workgroups of k_clear for n elements
template <typename T>
inline unsigned clear_blocks(long long n) {
    const long long per_block = 256 * (16 / (long long)sizeof(T));
    return (unsigned)((n + per_block - 1) / per_block);
}

}  // namespace tad
