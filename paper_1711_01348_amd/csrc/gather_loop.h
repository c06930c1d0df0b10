// Nested loops over the kernel coordinates z of one gradient element (final formula of Sec. 5.1): ranges from the
// plan's Fourier-Motzkin rows, outermost coordinate z_{kappa-1} first.  The loops can be shared by `parts`
// cooperating threads (all of them call with the same element):
//   - one coordinate: the threads take its values in turn (thread `part` takes every parts-th value, so that the
//     threads of a wavefront read neighbouring elements together);
//   - several, and the outermost has at least parts / 8 values: thread `part` takes every parts-th of them;
//   - otherwise every thread walks the outer coordinates, the values of an innermost run of at least `parts`
//     values are taken in turn, and shorter runs are dealt out whole to the threads in turn (a short outer range
//     over long inner runs would leave most threads idle the other way).
// `run(z, count, step)` is called once per innermost run with z[0] at the caller's first value; it handles the
// `count` values z[0], z[0] + step, ... itself (offsets advance by a constant per value there).
#pragma once
#include <hip/hip_runtime.h>

#include "plan_dev.h"

namespace tad {

template <class Run>
__device__ __forceinline__ void gather_loops(const GatherPlan &P, const int32_t *y, int part, int parts, Run &&run) {
    // `run` is expanded in line: the walk below is arranged so that it is called from one place only
    int32_t z[kMaxKernel] = {0, 0, 0, 0}, hi[kMaxKernel] = {0, 0, 0, 0};
    const int top = P.kappa - 1;
    bool single = false;       // exactly one run: no coordinate at all, or one coordinate shared by the threads
    bool share_runs = false;   // the same for all cooperating threads: the top range depends on the element only
    int32_t count = 1, step = 1;
    int step_top = 1;
    if (P.kappa == 0) {
        if (part != 0) return;   // a single term: z is empty
        single = true;
    } else {
        gather_bounds(P, top, y, z, z[top], hi[top]);
        if (parts > 1) {
            if (top == 0) {
                const int64_t first = (int64_t)z[0] + part;
                if (first > hi[0]) return;
                z[0] = (int32_t)first;
                count = (int32_t)((hi[0] - first) / parts + 1);
                step = parts;
                single = true;
            } else if (((int64_t)hi[top] - z[top] + 1) * 8 >= parts) {
                z[top] += part;
                step_top = parts;
            } else {
                share_runs = true;
            }
        }
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
                    z[lvl] += lvl == top ? step_top : 1;
                } else if (lvl == 0) {
                    break;
                } else {
                    --lvl;
                    gather_bounds(P, lvl, y, z, z[lvl], hi[lvl]);
                }
            }
            count = hi[0] - z[0] + 1;   // >= 1 here
            step = 1;
            if (share_runs) {
                if (count >= parts) {
                    z[0] += part;
                    count = (hi[0] - z[0]) / parts + 1;
                    step = parts;
                } else {
                    mine = turn == part;
                    turn = turn + 1 == parts ? 0 : turn + 1;
                }
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

// The cooperative form (one block per gradient element) pays off when an element sums many terms: measured on the
// worked expression at 8192 x 8192 x 5, the gradients with 8192 and 40960 terms per element take 0.8 ms this way
// against 11 ms with one thread per element.
inline bool use_cooperative_gather(long long n_elements, double terms_total) {
    return n_elements <= (1ll << 22) && terms_total / (double)(n_elements > 0 ? n_elements : 1) >= 1024.0;
}

}  // namespace tad
