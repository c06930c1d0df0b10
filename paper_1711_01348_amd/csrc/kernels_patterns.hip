// Specialised fp32 kernels for the three index patterns of the paper's introduction (Sec. 1), for any
// one-argument body without an inner sum, f = phi(x):
//
//   row reduce     f_ij = phi(x_i)       dx_i  = phi'(x_i) sum_j df_ij           (the index j collapses)
//   diagonal       f_i  = phi(x_ii)      dx_ij = delta_ij df_i phi'(x_ii)        (cokernel mask, no sum)
//   antidiagonal   f_ij = phi(x_{i+j})   dx_m  = phi'(x_m) sum_{i in window(m)} df_{i,m-i}
//
// Masks and the window come from the derived plan (gather_prepare / gather_bounds); the kernels only add
// the memory mapping: wide coalesced streams, wavefront reductions, per-tile partials finished in fixed order.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "bodies.h"
#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "launch_geom.h"

namespace tad {

typedef float float4v __attribute__((ext_vector_type(4)));

template <int BODY> __device__ __forceinline__ float phi(float x) { return body_outer<BODY, float>(x); }
// phi'(x), with f = phi(x) available for bodies whose derivative is expressed through f
template <int BODY> __device__ __forceinline__ float dphi(float x) {
    float v[1] = {x};
    return body_douter<BODY, float>(BODY == TAD_BODY_EXP ? phi<BODY>(x) : 0.f, v);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_p(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, ROW_MASK == 0xf);
    return v + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum63(float v) {   // total valid in lane 63
    v = dpp_add_p<0x111, 0xf>(v);
    v = dpp_add_p<0x112, 0xf>(v);
    v = dpp_add_p<0x114, 0xf>(v);
    v = dpp_add_p<0x118, 0xf>(v);
    v = dpp_add_p<0x142, 0xa>(v);
    v = dpp_add_p<0x143, 0xc>(v);
    return v;
}

// ------------------------------------------------------------------------------------------------
// row reduce
// ------------------------------------------------------------------------------------------------

// block: 1024 columns x RR_FTI rows, lane owns 4 consecutive columns
constexpr int RR_FTI = 2;
template <int BODY>
__global__ __launch_bounds__(256) void k_rowreduce_forward(const float *__restrict__ x, float *__restrict__ f,
                                                           int I, int J) {
    const int j0 = blockIdx.x * 1024 + threadIdx.x * 4;
    const int i0 = blockIdx.y * RR_FTI;
    if (j0 >= J) return;
    const int rows = min(RR_FTI, I - i0);
    float *fp = f + (size_t)i0 * J + j0;
    for (int r = 0; r < rows; ++r) {
        const float v = phi<BODY>(x[i0 + r]);
        float4v o = {v, v, v, v};
        __builtin_nontemporal_store(o, reinterpret_cast<float4v *>(fp));
        fp += J;
    }
}

// one block per row of df (four waves share the row; the j range of the plan is the whole row: collapsed kernel
// coordinate); y = beta for this family (checked on the host), the feasibility rows zero the elements of a longer x.
// Many small blocks: a 64 MiB read is too short for fewer, longer-running waves to reach the streaming rate.
template <int BODY>
__global__ __launch_bounds__(256) void k_rowreduce_backward(const FlatFeas feas, const float *__restrict__ x,
                                                            const float *__restrict__ df, float *__restrict__ dx,
                                                            int n_x, int J) {
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = blockIdx.x;
    const int32_t y[3] = {i, 0, 0};
    if (!flat_feasible(feas, y)) {   // uniform over the block
        if (tid == 0) dx[i] = 0.f;
        return;
    }
    const float *row = df + (size_t)i * J;
    float4v acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};
    int j = tid * 4;
    for (; j + 3 * 1024 < J; j += 4 * 1024) {
        float4v v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4v *>(row + j + u * 1024);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] += v[u];
    }
    for (; j < J; j += 1024) acc[0] += *reinterpret_cast<const float4v *>(row + j);
    const float4v t = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    const float s = wave_sum63((t[0] + t[1]) + (t[2] + t[3]));
    if (lane == 63) red[wave] = s;
    __syncthreads();
    if (tid == 0) dx[i] = dphi<BODY>(x[i]) * ((red[0] + red[1]) + (red[2] + red[3]));
}

// ------------------------------------------------------------------------------------------------
// diagonal
// ------------------------------------------------------------------------------------------------

template <int BODY>
__global__ __launch_bounds__(256) void k_diagonal_forward(const float *__restrict__ x, float *__restrict__ f,
                                                          int I, int ld) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < I) f[i] = phi<BODY>(x[(size_t)i * ld + i]);
}

// dense write of dx (rows x ld): zeros, except where the plan's masks pass (the diagonal inside the range)
// block: 1024 columns x DG_TI rows
constexpr int DG_TI = 2;
template <int BODY>
__global__ __launch_bounds__(256) void k_diagonal_backward(const FlatFeas feas, const float *__restrict__ x,
                                                           const float *__restrict__ df, float *__restrict__ dx,
                                                           int rows, int ld) {
    const int c0 = blockIdx.x * 1024 + threadIdx.x * 4;
    const int r0 = blockIdx.y * DG_TI;
    if (c0 >= ld) return;
    const int nr = min(DG_TI, rows - r0);
    for (int r = 0; r < nr; ++r) {
        const int row = r0 + r;
        float4v o = {0.f, 0.f, 0.f, 0.f};
        if (row >= c0 && row < c0 + 4) {
            // on the diagonal the cokernel condition holds; the transformed index is y = row (checked on the
            // host); the feasibility rows remove rows beyond the range of f
            const int32_t y[3] = {row, 0, 0};
            if (flat_feasible(feas, y)) {
                const float xv = x[(size_t)row * ld + row];
                o[row - c0] = df[row] * dphi<BODY>(xv);
            }
        }
        __builtin_nontemporal_store(o, reinterpret_cast<float4v *>(dx + (size_t)row * ld + c0));
    }
}

// ------------------------------------------------------------------------------------------------
// antidiagonal
// ------------------------------------------------------------------------------------------------
constexpr int AD_FTI = 32;    // rows per forward block
constexpr int AD_BTI = AD_BTI_ROWS;    // rows per backward tile

// block: 1024 columns x AD_FTI rows; the lane's window of phi(x) slides by one element per row
template <int BODY>
__global__ __launch_bounds__(256) void k_antidiag_forward(const float *__restrict__ x, float *__restrict__ f,
                                                          int I, int J) {
    const int j0 = blockIdx.x * 1024 + threadIdx.x * 4;
    const int i0 = blockIdx.y * AD_FTI;
    if (j0 >= J) return;
    const int rows = min(AD_FTI, I - i0);
    const float *xp = x + i0 + j0;
    float4v e = {phi<BODY>(xp[0]), phi<BODY>(xp[1]), phi<BODY>(xp[2]), phi<BODY>(xp[3])};
    float *fp = f + (size_t)i0 * J + j0;
    for (int r = 0; r < rows; ++r) {
        __builtin_nontemporal_store(e, reinterpret_cast<float4v *>(fp));
        fp += J;
        if (r + 1 < rows) {
            const float nx = phi<BODY>(xp[r + 4]);   // i0 + r + 1 + j0 + 3 <= I + J - 2: inside x
            e = float4v{e[1], e[2], e[3], nx};
        }
    }
}

// partial[tile][m] = sum over the rows i of the tile that lie in window(m) of df[i][m - i].
// Thread owns m: for a fixed row consecutive m are consecutive addresses.  z is the plan's kernel coordinate,
// i = iy*y + iz*z (iz = +-1), j = jy*y + jz*z.
__global__ __launch_bounds__(256) void k_antidiag_backward(const FlatFeas feas, const FlatLevel win, int iy, int iz,
                                                           int jy, int jz, const float *__restrict__ df,
                                                           float *__restrict__ part, int n_x, int J) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= n_x) return;
    const int t = blockIdx.y;
    const int32_t y[3] = {m, 0, 0};   // the transformed index is the gradient index (checked on the host)
    float s = 0.f;
    if (flat_feasible(feas, y)) {
        int32_t lo, hi;
        flat_bounds(win, y, lo, hi);
        // rows of this tile: i0 <= iy*y + iz*z < i0 + AD_BTI
        const int base = iy * y[0], i0 = t * AD_BTI;
        int zlo, zhi;
        if (iz > 0) { zlo = i0 - base; zhi = i0 + AD_BTI - 1 - base; }
        else { zlo = base - (i0 + AD_BTI - 1); zhi = base - i0; }
        lo = max(lo, zlo);
        hi = min(hi, zhi);
        const long long step = (long long)iz * J + jz;
        const float *p = df + ((long long)(base + iz * lo) * J + (jy * y[0] + jz * lo));
        // four loads in flight per lane; measured faster than 8 or 16 (also with the surplus ones switched off), than
        // non-temporal loads, and than 64-column blocks whose four waves split the rows
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        int w = lo;
        for (; w + 3 <= hi; w += 4) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = p[u * step];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] += v[u];
            p += 4 * step;
        }
        for (; w <= hi; ++w) { acc[0] += *p; p += step; }
        s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    }
    part[(size_t)t * n_x + m] = s;
}

// 64 outputs per block; sixteen waves split the tiles (a short chain of independent loads per thread) and are
// combined in fixed order
constexpr int AD_FIN_WAVES = 16;
template <int BODY>
__global__ __launch_bounds__(64 * AD_FIN_WAVES) void k_antidiag_finish(const float *__restrict__ x,
                                                                       const float *__restrict__ part, int n_tiles,
                                                                       float *__restrict__ dx, int n_x) {
    __shared__ double red[AD_FIN_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = blockIdx.x * 64 + lane;
    double s = 0.0;
    if (m < n_x) {
        int t = wave;
        for (; t + 3 * AD_FIN_WAVES < n_tiles; t += 4 * AD_FIN_WAVES) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = part[(size_t)(t + u * AD_FIN_WAVES) * n_x + m];
#pragma unroll
            for (int u = 0; u < 4; ++u) s += (double)v[u];
        }
        for (; t < n_tiles; t += AD_FIN_WAVES) s += (double)part[(size_t)t * n_x + m];
    }
    red[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && m < n_x) {
        s = 0.0;
#pragma unroll
        for (int w = 0; w < AD_FIN_WAVES; ++w) s += red[w][lane];
        dx[m] = (float)((double)dphi<BODY>(x[m]) * s);
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------

#define TAD_UNARY_SWITCH(body, CALL)                                   \
    switch (body) {                                                    \
    case TAD_BODY_SQ: { constexpr int B_ = TAD_BODY_SQ; CALL; break; }       \
    case TAD_BODY_CUBE: { constexpr int B_ = TAD_BODY_CUBE; CALL; break; }   \
    case TAD_BODY_SIN: { constexpr int B_ = TAD_BODY_SIN; CALL; break; }     \
    case TAD_BODY_EXP: { constexpr int B_ = TAD_BODY_EXP; CALL; break; }     \
    default: return TAD_EUNSUPPORTED;                                  \
    }

int pattern_forward(const tad_plan &pl, const void *const *args, void *fo, hipStream_t s) {
    const float *x = (const float *)args[0];
    float *f = (float *)fo;
    const int I = (int)pl.fast.I, J = (int)pl.fast.J;
    switch (pl.fwd_family) {
    case TAD_FAMILY_ROW_REDUCE:
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_rowreduce_forward", (k_rowreduce_forward<B_>),
                                                  dim3((J + 1023) / 1024, (I + RR_FTI - 1) / RR_FTI), dim3(256), 0, s, x, f, I, J));
        break;
    case TAD_FAMILY_DIAGONAL:
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_diagonal_forward", (k_diagonal_forward<B_>),
                                                  dim3((I + 255) / 256), dim3(256), 0, s, x, f, I, (int)pl.fast.c_ld));
        break;
    case TAD_FAMILY_ANTIDIAGONAL:
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_antidiag_forward", (k_antidiag_forward<B_>),
                                                  dim3((J + 1023) / 1024, (I + AD_FTI - 1) / AD_FTI), dim3(256), 0, s,
                                                  x, f, I, J));
        break;
    default: return TAD_EUNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

int pattern_backward(const tad_plan &pl, const void *const *args, const void *df_, void *const *dx_, void *ws,
                     hipStream_t s) {
    if (!dx_[0]) return TAD_OK;
    const float *x = (const float *)args[0], *df = (const float *)df_;
    float *dx = (float *)dx_[0];
    const int I = (int)pl.fast.I, J = (int)pl.fast.J;
    const int n_x = (int)pl.arg_count[0];
    switch (pl.ap[0].family) {
    case TAD_FAMILY_ROW_REDUCE:
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_rowreduce_backward", (k_rowreduce_backward<B_>),
                                                  dim3(n_x), dim3(256), 0, s, pl.fast.feas, x, df, dx,
                                                  n_x, J));
        break;
    case TAD_FAMILY_DIAGONAL: {
        const int rows = (int)pl.args[0].shape[0], ld = (int)pl.args[0].shape[1];
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_diagonal_backward", (k_diagonal_backward<B_>),
                                                  dim3((ld + 1023) / 1024, (rows + DG_TI - 1) / DG_TI), dim3(256), 0, s,
                                                  pl.fast.feas, x, df, dx, rows, ld));
        break;
    }
    case TAD_FAMILY_ANTIDIAGONAL: {
        const int n_tiles = (I + AD_BTI - 1) / AD_BTI;
        float *part = (float *)ws;
        TAD_LAUNCH("k_antidiag_backward", k_antidiag_backward, dim3((n_x + 255) / 256, n_tiles), dim3(256), 0, s,
                   pl.fast.feas, pl.fast.flat[0], pl.fast.dd_iy, pl.fast.dd_iz, pl.fast.jy, pl.fast.jz, df, part, n_x,
                   J);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_antidiag_finish", (k_antidiag_finish<B_>),
                                                  dim3((n_x + 63) / 64), dim3(64 * AD_FIN_WAVES), 0, s, x, part, n_tiles, dx, n_x));
        break;
    }
    default: return TAD_EUNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

}  // namespace tad
