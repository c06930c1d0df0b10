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

#include <algorithm>

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

__global__ __launch_bounds__(256) void k_strided_forward_direct(const StridedGeom g, const float *__restrict__ x,
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
__global__ __launch_bounds__(256) void k_strided_backward_direct(const StridedGeom g, const StridedDx D,
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

// ------------------------------------------------------------------------------------------------
// Tiled kernels.  The index maps of this family make whole-row pieces of the tensors contiguous: the rows of x that
// a few rows i of f read, and the rows of f that the gradient of a few rows p of x sums over.  A block stages such a
// slice in LDS once, with aligned 16-byte loads, and every term is then an LDS read.
//
// These kernels run a few microseconds, and a wavefront that walks once through a long stretch of code waits for
// its instructions more than for its data (about 200 cycles per 64 bytes of code never executed before on that
// compute unit): everything that repeats is a loop that is not unrolled, the plan's range rows are evaluated by one
// copy of the row arithmetic, and nothing is specialised that a loop bound can express.
// ------------------------------------------------------------------------------------------------

typedef float float4s __attribute__((ext_vector_type(4)));

struct LoadPlain {      // the tensor itself
    const float *__restrict__ p;
    __device__ __forceinline__ float4s four(int at) const { return *reinterpret_cast<const float4s *>(p + at); }
    __device__ __forceinline__ float one(int at) const { return p[at]; }
};
struct LoadSeed {       // t = df (1 - f^2), the factor every term of both gradients shares
    const float *__restrict__ f, *__restrict__ df;
    __device__ __forceinline__ float4s four(int at) const {
        const float4s a = *reinterpret_cast<const float4s *>(f + at), d = *reinterpret_cast<const float4s *>(df + at);
        return d * (1.f - a * a);
    }
    __device__ __forceinline__ float one(int at) const { const float a = f[at]; return df[at] * (1.f - a * a); }
};

// Floats [first, first + count) of a tensor of `limit` floats -> lds[mis + k] for element first + k, copied by the NT
// threads tid = 0 .. NT-1, where mis
// (returned) is the distance of the first element from the 16-byte boundary below it.  Vectors that lie inside the
// tensor are loaded whole, four per thread in flight; the at most two vectors that stick out, element by element.
template <int NT, class OP>
__device__ __forceinline__ int slice_to_lds(const float *__restrict__ base, int first, int count, int limit, float *lds,
                                            int tid, OP op) {
    const int mis = (int)((reinterpret_cast<uintptr_t>(base + first) >> 2) & 3);
    const int start = first - mis;                       // tensor index of lds[0] (tensors hold fewer than 2^31 elements)
    const int nvec = (mis + count + 3) >> 2;
TAD_NOUNROLL
    for (int v0 = tid; v0 < nvec; v0 += 4 * NT) {
        float4s val[4];
        bool inside[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int v = v0 + h * NT;
            const int at = start + 4 * v;
            inside[h] = v < nvec && at >= 0 && at <= limit - 4;
            if (inside[h]) val[h] = op.four(at);
        }
#pragma unroll
        for (int h = 0; h < 4; ++h)
            if (inside[h]) *reinterpret_cast<float4s *>(lds + 4 * (v0 + h * NT)) = val[h];
    }
    // the first and the last vector may reach beyond the tensor: their elements one by one (zeros outside)
    if (tid < 8) {
        const int v = tid < 4 ? 0 : nvec - 1, c = tid & 3;
        const int at = start + 4 * v;
        if (at < 0 || at > limit - 4) lds[4 * v + c] = (at + c >= 0 && at + c < limit) ? op.one(at + c) : 0.f;
    }
    return mis;
}

// forward: block = `ti` rows i of one n; the rows s*i0 .. s*(i0+rows-1)+U-1 of x[n] are one contiguous slice
__global__ __launch_bounds__(256) void k_strided_forward(const StridedGeom g, int ti, const float *__restrict__ x,
                                                         const float *__restrict__ w, float *__restrict__ f) {
    extern __shared__ float4s dyn4[];
    float *xs = reinterpret_cast<float *>(dyn4);
    __shared__ float ws[kMaxTaps];
    const int n_it = (g.I + ti - 1) / ti;
    const int n = blockIdx.x / n_it, i0 = (blockIdx.x % n_it) * ti;
    const int rows = min(ti, g.I - i0);
    if (threadIdx.x < g.U * g.V) ws[threadIdx.x] = w[threadIdx.x];
    const int mis = slice_to_lds<256>(x, (n * g.P + g.s * i0) * g.Q, (g.s * (rows - 1) + g.U) * g.Q, g.N * g.P * g.Q, xs,
                                      (int)threadIdx.x, LoadPlain{x});
    __syncthreads();
    float *out = f + ((size_t)n * g.I + i0) * g.J;
    const int ne = rows * g.J;
    int il = 0, j = threadIdx.x;
TAD_NOUNROLL
    for (int e = threadIdx.x; e < ne; e += 256) {
        while (j >= g.J) { j -= g.J; ++il; }
        const float *xp = xs + mis + (g.s * il) * g.Q + g.s * j;
        float acc = 0.f;
TAD_NOUNROLL
        for (int u = 0; u < g.U; ++u) {
TAD_NOUNROLL
            for (int v = 0; v < g.V; ++v) acc = fmaf(xp[u * g.Q + v], ws[u * g.V + v], acc);
        }
        out[e] = tanhf(acc);
        j += 256;
    }
}

// minimum / maximum over the wavefront with DPP moves (no LDS round trips); the result is valid in lane 63 and
// returned as a wave-uniform value
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_other(int v) {   // lanes without a source keep their own value
    return __builtin_amdgcn_update_dpp(v, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_min(int v) {
    v = min(v, dpp_other<0x111, 0xf>(v));
    v = min(v, dpp_other<0x112, 0xf>(v));
    v = min(v, dpp_other<0x114, 0xf>(v));
    v = min(v, dpp_other<0x118, 0xf>(v));
    v = min(v, dpp_other<0x142, 0xa>(v));
    v = min(v, dpp_other<0x143, 0xc>(v));
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_max(int v) { return -wave_min(-v); }

// Block roles in one launch.
//  * blocks [0, blocks_dw): dw over `ti` rows i of one n.  The slice of x those rows read sits in LDS; a thread owns up
//    to kStridedMaxPerThread function elements, whose t = df (1 - f^2) it loads before the slice is staged; wavefront
//    (DPP) and block reduction to part[block][taps].
//  * blocks [blocks_dw, ...): dx.  Each wavefront works on its own: `tp` rows p of one n, 64 columns q.  The plan gives
//    every element its masks and its two ranges (feasibility rows, rational range rows rounded exactly).  Each range
//    depends on one component of beta only (checked on the host: `rowlvl` is the level that moves with p, the other
//    one moves with q), so the wavefront evaluates the range rows once per column (lane = column) and once per row
//    (lane = row), twelve exact divisions each, instead of once per element; both stay in registers.  The offsets of
//    f that the terms reach form an interval (a wave-wide min / max); t on it is staged in the wavefront's piece of
//    LDS.  An interval longer than that piece is read from memory instead (slow, but nothing relies on the size).
//    Then the lanes walk the rows: the row range is the same for the whole wavefront (read from its lane).
template <int TAPS>
__global__ __launch_bounds__(256) void k_strided_backward(const StridedGeom g, const StridedDx D, int ti, int tp, int t_cap,
                                                          int rowlvl, int has_feas,
                                                          const float *__restrict__ x, const float *__restrict__ w,
                                                          const float *__restrict__ f, const float *__restrict__ df,
                                                          float *__restrict__ dx, float *__restrict__ part, int blocks_dw) {
    extern __shared__ float4s dyn4[];
    float *lds = reinterpret_cast<float *>(dyn4);
    __shared__ float ws[kMaxTaps];
    __shared__ float red[4][TAPS];
    __shared__ int tapoff[TAPS];
    const int taps = g.U * g.V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)blockIdx.x >= blocks_dw) {
        // ---------------- dx: one wavefront per work item (n, tp rows p, 64 columns q) ----------------
        const int n_cs = (g.Q + 63) >> 6, n_pt = (g.P + tp - 1) / tp;
        const int item = __builtin_amdgcn_readfirstlane((((int)blockIdx.x - blocks_dw) << 2) + wave);
        const bool have = item < g.N * n_pt * n_cs;
        const int cs = item % n_cs, pt = (item / n_cs) % n_pt, n = have ? item / (n_cs * n_pt) : 0;
        const int p0 = pt * tp, rows = min(tp, g.P - p0), q = (cs << 6) + lane;
        const bool active = have && q < g.Q;
        if (threadIdx.x < taps) ws[threadIdx.x] = w[threadIdx.x];
        const int fZr = D.fZ[rowlvl], fZc = D.fZ[1 - rowlvl], wZr = D.wZ[rowlvl], wZc = D.wZ[1 - rowlvl];
        // The range that moves with the column, for this lane's column, and the range that moves with the row, in lane
        // r for row p0 + r, from the range rows in the kernel arguments (no memory access).  Feasibility rows
        // (Sec. 4.2) that do not move with q belong to the rows, those that move with q alone to the columns: a failed
        // row empties the range.  Rows that mix q with n or p are left to the elements (has_feas).
        int32_t clo = 0, chi = -1, rlo = 0, rhi = -1;
        {
            const int32_t y[3] = {n, 0, q};
            int32_t lo, hi;
            flat_bounds(D.lvl[1 - rowlvl], y, lo, hi);
            bool ok = active;
#pragma unroll
            for (int r = 0; r < kFlatFeas; ++r)
                if (D.feas.ky[r][2] != 0 && D.feas.ky[r][0] == 0 && D.feas.ky[r][1] == 0)
                    ok = ok && D.feas.k0[r] + mul24(D.feas.ky[r][2], q) <= 0;
            if (ok) { clo = lo; chi = hi; }
        }
        {
            const int32_t y[3] = {n, p0 + lane, 0};
            int32_t lo, hi;
            flat_bounds(D.lvl[rowlvl], y, lo, hi);
            bool ok = have && lane < rows;
#pragma unroll
            for (int r = 0; r < kFlatFeas; ++r)
                if (D.feas.ky[r][2] == 0)
                    ok = ok && D.feas.k0[r] + mul24(D.feas.ky[r][0], y[0]) + mul24(D.feas.ky[r][1], y[1]) <= 0;
            if (ok) { rlo = lo; rhi = hi; }
        }
        // the offsets of f that the terms of this work item reach lie in one interval: extremes of the linear part
        // over the item's rows and columns plus those of the two range parts
        const bool cany = clo <= chi, rany = rlo <= rhi;
        const int cmin = wave_min(cany ? min(fZc * clo, fZc * chi) : INT32_MAX);
        const int cmax = wave_max(cany ? max(fZc * clo, fZc * chi) : -INT32_MAX);
        const int rmin = wave_min(rany ? min(fZr * rlo, fZr * rhi) : INT32_MAX);
        const int rmax = wave_max(rany ? max(fZr * rlo, fZr * rhi) : -INT32_MAX);
        const int nmax = wave_max(cany ? chi - clo + 1 : 0), rlen = wave_max(rany ? rhi - rlo + 1 : 0);
        const int q_a = cs << 6, q_b = min(q_a + 63, g.Q - 1);
        const int b1a = D.fY[1] * p0, b1b = D.fY[1] * (p0 + rows - 1), b2a = D.fY[2] * q_a, b2b = D.fY[2] * q_b;
        const bool none = cmin > cmax || rmin > rmax;
        const int omin = none ? 0 : D.fY[0] * n + min(b1a, b1b) + min(b2a, b2b) + rmin + cmin;
        const int omax = none ? -1 : D.fY[0] * n + max(b1a, b1b) + max(b2a, b2b) + rmax + cmax;
        const bool staged = !none && omin >= 0 && omax - omin + 1 + 8 <= t_cap;   // uniform over the wavefront
        float *slice = lds + wave * t_cap;
        int shift = 0;                                                   // slice[shift + of] = t at offset of
        if (staged)
            shift = slice_to_lds<64>(f, omin, omax - omin + 1, g.N * g.I * g.J, slice, lane, LoadSeed{f, df}) - omin;
        __syncthreads();
        float *out = dx + ((size_t)n * g.P + p0) * g.Q + q;
        const int col_f = D.fY[0] * n + D.fY[2] * q + shift, col_w = D.wY[0] * n + D.wY[2] * q;
        int pr_done = 0;
        if (staged && nmax <= 2 && rlen <= 2 && !has_feas) {
            // At most two values in either range (a stride of two or more under a 3 x 3 filter, ...).  What a term
            // takes from the column is the same in every row and stays in registers: its part of the two LDS
            // addresses and whether it exists.  What it takes from the row is the same for all lanes (scalars).  Four
            // rows at a time: their 32 LDS reads are issued together and waited for once.  A term that does not exist
            // reads where its neighbour lies and counts zero.
            int cf[2], cw[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const bool cvb = clo + b <= chi;
                cf[b] = col_f + fZc * (cvb ? clo + b : clo);
                cw[b] = col_w + wZc * (cvb ? clo + b : clo);
            }
            const bool lane_any = cany, second = clo + 1 <= chi;
TAD_NOUNROLL
            for (; pr_done + 4 <= rows; pr_done += 4) {
                int r_lo[4], r_hi[4];
                bool whole = true;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    r_lo[u] = __builtin_amdgcn_readlane(rlo, pr_done + u);
                    r_hi[u] = __builtin_amdgcn_readlane(rhi, pr_done + u);
                    whole = whole && r_lo[u] <= r_hi[u];
                }
                if (!whole) break;                         // a row without terms: the plain loop below takes over
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
                if (lane_any) {                            // lanes without any term stay out of LDS
                    float t[4][2][2], wv[4][2][2];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int a = 0; a < 2; ++a) {
                            const int zr = a <= r_hi[u] - r_lo[u] ? r_lo[u] + a : r_lo[u];
                            const int rf = D.fY[1] * (p0 + pr_done + u) + fZr * zr, rw = D.wY[1] * (p0 + pr_done + u) + wZr * zr;
#pragma unroll
                            for (int b = 0; b < 2; ++b) {
                                t[u][a][b] = slice[cf[b] + rf];
                                wv[u][a][b] = ws[cw[b] + rw];
                            }
                        }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int a = 0; a < 2; ++a) {
                            const float m = a <= r_hi[u] - r_lo[u] ? 1.f : 0.f;     // the same for all lanes
                            float part = t[u][a][0] * wv[u][a][0];
                            part = fmaf(second ? t[u][a][1] : 0.f, wv[u][a][1], part);
                            acc[u] = fmaf(m, part, acc[u]);
                        }
                }
                if (active) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) out[(size_t)(pr_done + u) * g.Q] = acc[u];
                }
            }
        }
TAD_NOUNROLL
        for (int pr = pr_done; pr < rows; ++pr) {      // rows the batched form has left, or all rows
            const int r_lo = __builtin_amdgcn_readlane(rlo, pr), r_hi = __builtin_amdgcn_readlane(rhi, pr);
            const int32_t y[3] = {n, p0 + pr, q};
            const bool ok = active && (!has_feas || flat_feasible(D.feas, y));
            const int base_f = col_f + D.fY[1] * y[1], base_w = col_w + D.wY[1] * y[1];
            float acc = 0.f;
TAD_NOUNROLL
            for (int zr = r_lo; zr <= r_hi; ++zr) {
TAD_NOUNROLL
                for (int k = 0; k < nmax; ++k) {
                    const int zc = clo + k;
                    if (ok && zc <= chi) {
                        const int of = base_f + fZr * zr + fZc * zc;
                        float t;
                        if (staged) t = slice[of];
                        else { const float fv = f[of]; t = df[of] * (1.f - fv * fv); }     // shift = 0 here
                        acc = fmaf(t, ws[base_w + wZr * zr + wZc * zc], acc);
                    }
                }
            }
            if (active) out[(size_t)pr * g.Q] = acc;
        }
        return;
    }
    // ---------------- dw ----------------
    const int blk = blockIdx.x;
    const int n_it = (g.I + ti - 1) / ti;
    const int n = blk / n_it, i0 = (blk % n_it) * ti;
    const int rows = min(ti, g.I - i0);
    const int ne = rows * g.J;                         // <= 256 * kStridedMaxPerThread (chosen on the host)
    const size_t fbase = ((size_t)n * g.I + i0) * g.J;
    float tv[kStridedMaxPerThread];
    {
        float fv[kStridedMaxPerThread], dv[kStridedMaxPerThread];
#pragma unroll
        for (int k = 0; k < kStridedMaxPerThread; ++k) {
            const int e = threadIdx.x + 256 * k;
            fv[k] = e < ne ? f[fbase + e] : 0.f;
            dv[k] = e < ne ? df[fbase + e] : 0.f;
        }
        if (threadIdx.x < taps) tapoff[threadIdx.x] = (threadIdx.x / g.V) * g.Q + (threadIdx.x % g.V);
        const int mis = slice_to_lds<256>(x, (n * g.P + g.s * i0) * g.Q, (g.s * (rows - 1) + g.U) * g.Q, g.N * g.P * g.Q,
                                          lds, (int)threadIdx.x, LoadPlain{x});
        lds += mis;
#pragma unroll
        for (int k = 0; k < kStridedMaxPerThread; ++k) tv[k] = dv[k] * (1.f - fv[k] * fv[k]);
    }
    __syncthreads();
    float acc[TAPS];
#pragma unroll
    for (int q = 0; q < TAPS; ++q) acc[q] = 0.f;
    int il = 0, j = threadIdx.x;
#pragma unroll
    for (int k = 0; k < kStridedMaxPerThread; ++k) {
        const int e = threadIdx.x + 256 * k;
        if (e < ne) {
            while (j >= g.J) { j -= g.J; ++il; }
            const float *xp = lds + (g.s * il) * g.Q + g.s * j;
#pragma unroll
            for (int q = 0; q < TAPS; ++q)
                if (q < taps) acc[q] = fmaf(tv[k], xp[tapoff[q]], acc[q]);
            j += 256;
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

// dw_q = sum over the per-block partials, fixed order; one block of four waves per tap
__global__ __launch_bounds__(256) void k_strided_finish(const float *__restrict__ part, int n_part, int taps,
                                                        float *__restrict__ dw) {
    __shared__ double red[4];
    const int q = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double s = 0.0;
    for (int b = threadIdx.x; b < n_part; b += 256) s += (double)part[(size_t)b * taps + q];
    for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) dw[q] = (float)((red[0] + red[1]) + (red[2] + red[3]));
}

static StridedGeom geom(const tad_plan &pl) {
    StridedGeom g;
    g.N = (int)pl.fast.N; g.I = (int)pl.fast.I; g.J = (int)pl.fast.J; g.U = (int)pl.fast.U; g.V = (int)pl.fast.V;
    g.s = (int)pl.fast.stride; g.P = (int)pl.fast.P; g.Q = (int)pl.fast.Q;
    return g;
}

static StridedTiling tiling(const tad_plan &pl) {
    return strided_tiling(pl.fast.N, pl.fast.I, pl.fast.J, pl.fast.U, pl.fast.stride, pl.fast.P, pl.fast.Q);
}

int strided_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s) {
    const int nf = (int)pl.f_count;
    const StridedTiling t = tiling(pl);
    if (t.ti) {
        const int blocks = (int)(pl.fast.N * ((pl.fast.I + t.ti - 1) / t.ti));
        TAD_LAUNCH("k_strided_forward", k_strided_forward, dim3(blocks), dim3(256), (size_t)t.x_slice * 4, s, geom(pl), t.ti,
                   (const float *)args[0], (const float *)args[1], (float *)f);
    } else {
        TAD_LAUNCH("k_strided_forward_direct", k_strided_forward_direct, dim3((nf + 255) / 256), dim3(256), 0, s, geom(pl),
                   (const float *)args[0], (const float *)args[1], (float *)f, nf);
    }
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

static StridedDx dx_plan(const tad_plan &pl) {
    StridedDx D;
    D.feas = pl.fast.feas;
    D.lvl[0] = pl.fast.flat[0];
    D.lvl[1] = pl.fast.flat[1];
    const GatherPlan &gp = pl.ap[0].dev;
    for (int c = 0; c < 3; ++c) { D.fY[c] = (int32_t)gp.offY[kSlotF][c]; D.wY[c] = (int32_t)gp.offY[1][c]; }
    for (int m = 0; m < 2; ++m) { D.fZ[m] = (int32_t)gp.offZ[kSlotF][m]; D.wZ[m] = (int32_t)gp.offZ[1][m]; }
    return D;
}

template <int TAPS>
static void launch_bwd_direct(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                              void *const *dx, void *ws, int blocks_dx, int blocks_dw, hipStream_t s) {
    TAD_LAUNCH("k_strided_backward_direct", (k_strided_backward_direct<TAPS>), dim3(blocks_dx + blocks_dw), dim3(256), 0, s,
               geom(pl), dx_plan(pl), (const float *)args[0], (const float *)args[1], (const float *)f, (const float *)df,
               (float *)dx[0], (float *)ws, (int)pl.arg_count[0], (int)pl.f_count, blocks_dw);
}

// Which of the two range levels can be tabulated per row p (component 1 of beta) while the other one is tabulated per
// column q (component 2): 1 or 0; -1 if a level moves with both (then the direct kernel evaluates every element).
static int row_level(const tad_plan &pl) {
    auto free_of = [](const FlatLevel &L, int c) {
        for (int r = 0; r < kFlatRows; ++r)
            if (L.lky[r][c] != 0 || L.hky[r][c] != 0) return false;
        return true;
    };
    const FlatLevel &l0 = pl.fast.flat[0], &l1 = pl.fast.flat[1];
    if (free_of(l1, 2) && free_of(l0, 1)) return 1;
    if (free_of(l0, 2) && free_of(l1, 1)) return 0;
    return -1;
}

// 1 when a feasibility row of the loop-free plan moves with q and with n or p at once: such a row cannot be folded
// into the per-row and per-column range tables and the kernel tests the rows for every element
static int has_feasibility_rows(const tad_plan &pl) {
    const FlatFeas &F = pl.fast.feas;
    for (int r = 0; r < kFlatFeas; ++r)
        if (F.ky[r][2] != 0 && (F.ky[r][0] != 0 || F.ky[r][1] != 0)) return 1;
    return 0;
}

template <int TAPS>
static void launch_bwd(const tad_plan &pl, const StridedTiling &t, int rowlvl, const void *const *args, const void *f,
                       const void *df, void *const *dx, void *ws, int blocks_dx, int blocks_dw, hipStream_t s) {
    const size_t lds = (size_t)std::max(blocks_dw ? t.x_slice : 0, blocks_dx ? 4 * t.t_slice : 0) * 4;   // dx: a piece per wavefront
    TAD_LAUNCH("k_strided_backward", (k_strided_backward<TAPS>), dim3(blocks_dx + blocks_dw), dim3(256), lds, s, geom(pl),
               dx_plan(pl), t.ti, t.tp, t.t_slice, rowlvl, has_feasibility_rows(pl), (const float *)args[0], (const float *)args[1], (const float *)f,
               (const float *)df, (float *)dx[0], (float *)ws, blocks_dw);
}

#define TAD_TAPS_SWITCH(taps, CALL)                                   \
    do {                                                              \
        if (taps <= 4) { constexpr int T_ = 4; CALL; }                \
        else if (taps <= 9) { constexpr int T_ = 9; CALL; }           \
        else if (taps <= 16) { constexpr int T_ = 16; CALL; }         \
        else if (taps <= 25) { constexpr int T_ = 25; CALL; }         \
        else { constexpr int T_ = kMaxTaps; CALL; }                   \
    } while (0)

int strided_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                     void *const *dx, void *ws, hipStream_t s) {
    const int nf = (int)pl.f_count;
    const int taps = (int)(pl.fast.U * pl.fast.V);
    const StridedTiling t = tiling(pl);
    int blocks_dw = 0;
    const int rowlvl = row_level(pl);
    if (t.ti && t.tp && rowlvl >= 0) {
        // dx: one wavefront per (n, tp rows, 64 columns), four to a block
        const long long items = pl.fast.N * ((pl.fast.P + t.tp - 1) / t.tp) * ((pl.fast.Q + 63) / 64);
        const int blocks_dx = dx[0] ? (int)((items + 3) / 4) : 0;
        blocks_dw = dx[1] ? (int)(pl.fast.N * ((pl.fast.I + t.ti - 1) / t.ti)) : 0;
        if (blocks_dx + blocks_dw == 0) return TAD_OK;
        TAD_TAPS_SWITCH(taps, (launch_bwd<T_>(pl, t, rowlvl, args, f, df, dx, ws, blocks_dx, blocks_dw, s)));
    } else {
        const int blocks_dx = dx[0] ? (int)((pl.arg_count[0] + 255) / 256) : 0;
        blocks_dw = dx[1] ? (nf + kStridedDwElems - 1) / kStridedDwElems : 0;
        if (blocks_dx + blocks_dw == 0) return TAD_OK;
        TAD_TAPS_SWITCH(taps, (launch_bwd_direct<T_>(pl, args, f, df, dx, ws, blocks_dx, blocks_dw, s)));
    }
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dx[1]) {
        TAD_LAUNCH("k_strided_finish", k_strided_finish, dim3(taps), dim3(256), 0, s, (const float *)ws, blocks_dw,
                   taps, (float *)dx[1]);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

}  // namespace tad
