// Nested loops over the kernel coordinates z of one gradient element (final formula of Sec. 5.1): ranges from the
// plan's Fourier-Motzkin rows, outermost coordinate z_{kappa-1} first.  The loops can be shared by `parts`
// cooperating threads: thread `part` takes every parts-th value of the outermost coordinate (kappa > 1) or one
// contiguous piece of the only range (kappa = 1).  `run(z, z0_hi)` is called once per innermost run with z[0] at
// its first value; it handles z[0]..z0_hi itself (offsets advance by a constant per step there).
#pragma once
#include <hip/hip_runtime.h>

#include "plan_dev.h"

namespace tad {

template <class Run>
__device__ __forceinline__ void gather_loops(const GatherPlan &P, const int32_t *y, int part, int parts, Run &&run) {
    int32_t z[kMaxKernel] = {0, 0, 0, 0}, hi[kMaxKernel] = {0, 0, 0, 0};
    if (P.kappa == 0) {
        if (part == 0) run(z, 0);   // a single term: z is empty
        return;
    }
    const int top = P.kappa - 1;
    gather_bounds(P, top, y, z, z[top], hi[top]);
    if (parts > 1) {
        if (top == 0) {
            const int64_t len = (int64_t)hi[0] - z[0] + 1;
            if (len <= 0) return;
            const int64_t chunk = (len + parts - 1) / parts;
            const int64_t lo = z[0] + chunk * part;
            hi[0] = (int32_t)(lo + chunk - 1 < hi[0] ? lo + chunk - 1 : hi[0]);
            if (lo > hi[0]) return;
            z[0] = (int32_t)lo;
        } else {
            z[top] += part;
        }
    }
    const int step_top = (parts > 1 && top > 0) ? parts : 1;
    int lvl = top;
    for (;;) {
        if (z[lvl] > hi[lvl]) {
            if (++lvl > top) break;
            z[lvl] += lvl == top ? step_top : 1;
            continue;
        }
        if (lvl == 0) {
            run(z, hi[0]);
            z[0] = hi[0] + 1;
        } else {
            --lvl;
            gather_bounds(P, lvl, y, z, z[lvl], hi[lvl]);
        }
    }
}

// Sum of one double per thread over the block (256 threads), fixed order; the total is returned to thread 0.
__device__ __forceinline__ double block_sum_256(double v, double *red /* [4] in LDS */) {
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// Cooperative form pays off when there are few gradient elements and many terms per element.
inline bool use_cooperative_gather(long long n_elements, double terms_total) {
    return n_elements <= 8192 && terms_total / (double)(n_elements > 0 ? n_elements : 1) >= 2048.0;
}

}  // namespace tad
