// Specialised fp32 kernels for a strided (non-unimodular looking) index map,
//
//     f_nij = tanh( sum_{u<U, v<V} x_{n, s i + u, s j + v} w_uv ),
//
// extended index (n, i, j, u, v).  With t_nij = df_nij (1 - f_nij^2):
//     dx_npq = sum over the plan's two kernel coordinates of t * w      (at most ceil(U/s) ceil(V/s) terms;
//              the ranges are the rational Fourier-Motzkin bounds, rounded exactly, clipped at the border)
//     dw_uv  = sum_{n,i,j} t_nij x_{n, s i + u, s j + v}                  (all three kernel coordinates collapse:
//              block-level reduction to per-block partials, finished in fixed order)
#include <hip/hip_runtime.h>

#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "launch_geom.h"

namespace tad {

constexpr int kMaxTaps = 49;   // U*V <= 7*7

struct StridedGeom {
    int N, I, J, U, V, s, P, Q;   // x is N x P x Q
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_s(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, ROW_MASK == 0xf);
    return v + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum63s(float v) {
    v = dpp_add_s<0x111, 0xf>(v);
    v = dpp_add_s<0x112, 0xf>(v);
    v = dpp_add_s<0x114, 0xf>(v);
    v = dpp_add_s<0x118, 0xf>(v);
    v = dpp_add_s<0x142, 0xa>(v);
    v = dpp_add_s<0x143, 0xc>(v);
    return v;
}

__global__ __launch_bounds__(256) void k_strided_forward(const StridedGeom g, const float *__restrict__ x,
                                                         const float *__restrict__ w, float *__restrict__ f,
                                                         int nf) {
    __shared__ float ws[kMaxTaps];
    if (threadIdx.x < g.U * g.V) ws[threadIdx.x] = w[threadIdx.x];
    __syncthreads();
    const int lin = blockIdx.x * 256 + threadIdx.x;
    if (lin >= nf) return;
    const int j = lin % g.J, i = (lin / g.J) % g.I, n = lin / (g.J * g.I);
    const float *xp = x + ((size_t)n * g.P + (size_t)g.s * i) * g.Q + (size_t)g.s * j;
    float acc = 0.f;
    for (int u = 0; u < g.U; ++u)
        for (int v = 0; v < g.V; ++v) acc = fmaf(xp[(size_t)u * g.Q + v], ws[u * g.V + v], acc);
    f[lin] = tanhf(acc);
}

// Everything the dx role needs from the plan of x, in loop-free form (y = beta for this family).
struct StridedDx {
    FlatFeas feas;
    FlatLevel lvl[2];
    int32_t fY[3], fZ[2];   // element offset of f / df:  fY . beta + fZ . z
    int32_t wY[3], wZ[2];   // element offset of w
};

// Block roles in one launch.
//  * blocks [blocks_dw, ...): one thread per gradient element (n, p, q) of x.  Masks and both ranges come from
//    the plan (feasibility rows, rational range rows rounded exactly); the two ranges do not depend on each other.
//  * blocks [0, blocks_dw) reduce dw over kStridedDwElems function elements each into part[block][taps].
template <int TAPS>
__global__ __launch_bounds__(256) void k_strided_backward(const StridedGeom g, const StridedDx D,
                                                          const float *__restrict__ x, const float *__restrict__ w,
                                                          const float *__restrict__ f, const float *__restrict__ df,
                                                          float *__restrict__ dx, float *__restrict__ part, int n_x,
                                                          int nf, int blocks_dw) {
    __shared__ float ws[kMaxTaps];
    __shared__ float red[4][TAPS];
    __shared__ int tapoff[TAPS];
    const int taps = g.U * g.V;
    // the few long-running dw blocks come first in launch order so that they overlap the dx stream
    if ((int)blockIdx.x >= blocks_dw) {
        const int lin = ((int)blockIdx.x - blocks_dw) * 256 + threadIdx.x;
        const bool inside = lin < n_x;
        const int q = lin % g.Q, t = lin / g.Q;
        const int32_t y[3] = {t / g.P, t % g.P, q};
        int32_t lo1 = 0, hi1 = -1, lo0 = 0, hi0 = -1;
        if (inside && flat_feasible(D.feas, y)) {
            flat_bounds(D.lvl[1], y, lo1, hi1);
            flat_bounds(D.lvl[0], y, lo0, hi0);
        }
        const int base_f = D.fY[0] * y[0] + D.fY[1] * y[1] + D.fY[2] * y[2];
        const int base_w = D.wY[0] * y[0] + D.wY[1] * y[1] + D.wY[2] * y[2];
        const int n1 = hi1 - lo1 + 1, n0 = hi0 - lo0 + 1;
        // Up to two values per coordinate (a stride of two or more under a 3 x 3 filter, ...): the loads of all
        // terms are issued together, before the filter taps are staged, so that the wavefront waits for memory
        // once instead of once per term.  Terms are added in the order of the loops below.
        const bool few = n1 <= 2 && n0 <= 2;
        float fv[2][2], dv[2][2];
        if (few) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const bool on = a < n1 && b < n0;
                    const int of = base_f + D.fZ[1] * (lo1 + a) + D.fZ[0] * (lo0 + b);
                    fv[a][b] = on ? f[of] : 0.f;
                    dv[a][b] = on ? df[of] : 0.f;
                }
        }
        if (threadIdx.x < taps) ws[threadIdx.x] = w[threadIdx.x];
        __syncthreads();
        if (!inside) return;
        float acc = 0.f;
        if (few) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    if (a < n1 && b < n0)
                        acc = fmaf(dv[a][b] * (1.f - fv[a][b] * fv[a][b]),
                                   ws[base_w + D.wZ[1] * (lo1 + a) + D.wZ[0] * (lo0 + b)], acc);
        } else {
            for (int32_t z1 = lo1; z1 <= hi1; ++z1) {
                int of = base_f + D.fZ[1] * z1 + D.fZ[0] * lo0;
                int ow = base_w + D.wZ[1] * z1 + D.wZ[0] * lo0;
                for (int32_t z0 = lo0; z0 <= hi0; ++z0) {
                    const float fval = f[of];
                    acc = fmaf(df[of] * (1.f - fval * fval), ws[ow], acc);
                    of += D.fZ[0];
                    ow += D.wZ[0];
                }
            }
        }
        dx[lin] = acc;
        return;
    }
    if (threadIdx.x < taps) tapoff[threadIdx.x] = (threadIdx.x / g.V) * g.Q + (threadIdx.x % g.V);
    __syncthreads();
    const int blk = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float acc[TAPS];
#pragma unroll
    for (int q = 0; q < TAPS; ++q) acc[q] = 0.f;
#pragma unroll
    for (int e = 0; e < kStridedDwElems / 256; ++e) {
        const int lin = blk * kStridedDwElems + e * 256 + threadIdx.x;
        if (lin < nf) {
            const int j = lin % g.J, i = (lin / g.J) % g.I, n = lin / (g.J * g.I);
            const float fv = f[lin];
            const float t = df[lin] * (1.f - fv * fv);
            const float *xp = x + ((size_t)n * g.P + (size_t)g.s * i) * g.Q + (size_t)g.s * j;
#pragma unroll
            for (int q = 0; q < TAPS; ++q)
                if (q < taps) acc[q] = fmaf(t, xp[tapoff[q]], acc[q]);
        }
    }
#pragma unroll
    for (int q = 0; q < TAPS; ++q) {
        const float sum = wave_sum63s(acc[q]);
        if (lane == 63) red[wave][q] = sum;
    }
    __syncthreads();
    if (threadIdx.x < taps)
        part[(size_t)blk * taps + threadIdx.x] =
            (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// dw_q = sum over the per-block partials, fixed order; one wave per tap
__global__ __launch_bounds__(64) void k_strided_finish(const float *__restrict__ part, int n_part, int taps,
                                                       float *__restrict__ dw) {
    const int q = blockIdx.x, lane = threadIdx.x;
    double s = 0.0;
    for (int b = lane; b < n_part; b += 64) s += (double)part[(size_t)b * taps + q];
    for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
    if (lane == 0) dw[q] = (float)s;
}

static StridedGeom geom(const tad_plan &pl) {
    StridedGeom g;
    g.N = (int)pl.fast.N; g.I = (int)pl.fast.I; g.J = (int)pl.fast.J; g.U = (int)pl.fast.U; g.V = (int)pl.fast.V;
    g.s = (int)pl.fast.stride; g.P = (int)pl.fast.P; g.Q = (int)pl.fast.Q;
    return g;
}

int strided_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s) {
    const int nf = (int)pl.f_count;
    TAD_LAUNCH("k_strided_forward", k_strided_forward, dim3((nf + 255) / 256), dim3(256), 0, s, geom(pl),
               (const float *)args[0], (const float *)args[1], (float *)f, nf);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

template <int TAPS>
static void launch_bwd(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                       void *const *dx, void *ws, int blocks_dx, int blocks_dw, hipStream_t s) {
    StridedDx D;
    D.feas = pl.fast.feas;
    D.lvl[0] = pl.fast.flat[0];
    D.lvl[1] = pl.fast.flat[1];
    const GatherPlan &gp = pl.ap[0].dev;
    for (int c = 0; c < 3; ++c) { D.fY[c] = (int32_t)gp.offY[kSlotF][c]; D.wY[c] = (int32_t)gp.offY[1][c]; }
    for (int m = 0; m < 2; ++m) { D.fZ[m] = (int32_t)gp.offZ[kSlotF][m]; D.wZ[m] = (int32_t)gp.offZ[1][m]; }
    TAD_LAUNCH("k_strided_backward", (k_strided_backward<TAPS>), dim3(blocks_dx + blocks_dw), dim3(256), 0, s,
               geom(pl), D, (const float *)args[0], (const float *)args[1], (const float *)f, (const float *)df,
               (float *)dx[0], (float *)ws, (int)pl.arg_count[0], (int)pl.f_count, blocks_dw);
}

int strided_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                     void *const *dx, void *ws, hipStream_t s) {
    const int nf = (int)pl.f_count;
    const int taps = (int)(pl.fast.U * pl.fast.V);
    const int blocks_dx = dx[0] ? (int)((pl.arg_count[0] + 255) / 256) : 0;
    const int blocks_dw = dx[1] ? (nf + kStridedDwElems - 1) / kStridedDwElems : 0;
    if (blocks_dx + blocks_dw == 0) return TAD_OK;
    if (taps <= 4) launch_bwd<4>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s);
    else if (taps <= 9) launch_bwd<9>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s);
    else if (taps <= 16) launch_bwd<16>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s);
    else if (taps <= 25) launch_bwd<25>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s);
    else launch_bwd<kMaxTaps>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dx[1]) {
        TAD_LAUNCH("k_strided_finish", k_strided_finish, dim3(taps), dim3(64), 0, s, (const float *)ws, blocks_dw,
                   taps, (float *)dx[1]);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

}  // namespace tad
