// Specialised fp32 kernels for the worked expression of the paper (Sec. 1, Sec. 6)
//
//     f_ij = exp(-sum_k((a_ik + b_jk)^2 c_ii + d_{i+k}^3)),      k < K, K small,
//
// and its four gather-form gradients.  With g_ij = df_ij f_ij the derived expressions
// (Sec. 6, with the factors that do not depend on the summed kernel coordinate pulled out) are
//     r_i   = sum_j g_ij                       P_ik = sum_j g_ij b_jk        Q_i = sum_j g_ij |b_j|^2
//     t_j   = sum_i c_ii g_ij                  T_jk = sum_i c_ii g_ij a_ik
//     da_ik = -2 c_ii (a_ik r_i + P_ik)        db_jk = -2 (T_jk + b_jk t_j)
//     dc_ii = -(|a_i|^2 r_i + 2 sum_k a_ik P_ik + Q_i),   zero off the diagonal (cokernel mask)
//     dd_m  = -3 d_m^2 sum_{i in window(m)} r_i            (window from the plan's range rows)
// One pass over df and f produces the row sums (collapsed kernel coordinate j) and the column sums
// (collapsed kernel coordinate i) together; both are finished from per-tile partials in a fixed
// order, so results are deterministic and need no atomics.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "worked_geom.h"

namespace tad {

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// ---------------------------------------------------------------------------------------------
// forward: block = 4 waves, 1024 columns x FWD_TI rows; lane owns 4 consecutive columns
// ---------------------------------------------------------------------------------------------

template <int K>
__global__ __launch_bounds__(256) void k_worked_forward(const float *__restrict__ a, const float *__restrict__ b,
                                                        const float *__restrict__ c, const float *__restrict__ d,
                                                        float *__restrict__ f, int I, int J, int c_ld) {
    constexpr int RW = K + 2;
    __shared__ float rd[FWD_TI][RW];
    const int tid = threadIdx.x;
    const int i0 = blockIdx.y * FWD_TI;
    const int j0 = blockIdx.x * 1024 + tid * 4;
    if (tid < FWD_TI) {
        int i = i0 + tid;
        if (i < I) {
            float D = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                rd[tid][k] = a[(size_t)i * K + k];
                float dv = d[i + k];
                D = fmaf(dv * dv, dv, D);
            }
            rd[tid][K] = -kLog2e * c[(size_t)i * c_ld + i];
            rd[tid][K + 1] = -kLog2e * D;
        }
    }
    __syncthreads();
    if (j0 >= J) return;
    float bj[4][K];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int k = 0; k < K; ++k) bj[v][k] = b[(size_t)(j0 + v) * K + k];   // J % 4 == 0: all four columns exist
    const int rows = min(FWD_TI, I - i0);
    float *fp = f + (size_t)i0 * J + j0;
    for (int r = 0; r < rows; ++r) {
        float ai[K];
#pragma unroll
        for (int k = 0; k < K; ++k) ai[k] = rd[r][k];
        const float cs = rd[r][K], Ds = rd[r][K + 1];
        float4v e;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                float t = ai[k] + bj[v][k];
                s = fmaf(t, t, s);
            }
            e[v] = __builtin_amdgcn_exp2f(fmaf(cs, s, Ds));
        }
        *reinterpret_cast<float4v *>(fp) = e;
        fp += J;
    }
}

// ---------------------------------------------------------------------------------------------
// backward main pass: block = 4 waves over the same 256 columns, BWD_TI rows (each wave a quarter)
// ---------------------------------------------------------------------------------------------

template <int K>
__global__ __launch_bounds__(256) void k_worked_backward(const float *__restrict__ a, const float *__restrict__ b,
                                                         const float *__restrict__ c, const float *__restrict__ f,
                                                         const float *__restrict__ df, float *__restrict__ dc,
                                                         long long dc_count, float *__restrict__ rowp,
                                                         float *__restrict__ colp, int I, int J, int c_ld) {
    constexpr int RW = K + 1;      // a_i0..a_i{K-1}, c_ii
    constexpr int RP = K + 2;      // row partials: r, P_0..P_{K-1}, Q
    constexpr int CP = K + 1;      // column partials: t, T_0..T_{K-1}
    __shared__ float rd[BWD_TI][RW];
    __shared__ float cred[4][CP][BWD_TJ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = blockIdx.y * BWD_TI;
    const int j0 = blockIdx.x * BWD_TJ + lane * 4;
    const int nblk = gridDim.x * gridDim.y, blk = blockIdx.y * gridDim.x + blockIdx.x;

    // this block's share of the dense zero fill of dc (its diagonal is written by the finishing kernel)
    if (dc) {
        long long n4 = dc_count >> 2;
        long long per = (n4 + nblk - 1) / nblk;
        long long lo = (long long)blk * per, hi = lo + per < n4 ? lo + per : n4;
        float4v z = {0.f, 0.f, 0.f, 0.f};
        for (long long q = lo + tid; q < hi; q += 256) reinterpret_cast<float4v *>(dc)[q] = z;
        if (blk == 0 && tid < (int)(dc_count & 3)) dc[(n4 << 2) + tid] = 0.f;
    }

    for (int t = tid; t < BWD_TI; t += 256) {
        int i = i0 + t;
        if (i < I) {
#pragma unroll
            for (int k = 0; k < K; ++k) rd[t][k] = a[(size_t)i * K + k];
            rd[t][K] = c[(size_t)i * c_ld + i];
        }
    }
    __syncthreads();

    const bool live = j0 < J;
    float bj[4][K], nb[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        nb[v] = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            bj[v][k] = live ? b[(size_t)(j0 + v) * K + k] : 0.f;
            nb[v] = fmaf(bj[v][k], bj[v][k], nb[v]);
        }
    }
    float tc[4] = {0.f, 0.f, 0.f, 0.f}, Tc[4][K];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int k = 0; k < K; ++k) Tc[v][k] = 0.f;

    constexpr int WR = BWD_TI / 4;
    const int r0 = wave * WR;
    const int rows = max(0, min(WR, I - (i0 + r0)));
    const float *fp = f + (size_t)(i0 + r0) * J + j0;
    const float *gp = df + (size_t)(i0 + r0) * J + j0;
    float *rp = rowp + ((size_t)blockIdx.x * I + (i0 + r0)) * RP;
    for (int r = 0; r < rows; ++r) {
        float4v fv = {0.f, 0.f, 0.f, 0.f}, dv = fv;
        if (live) {
            fv = *reinterpret_cast<const float4v *>(fp);
            dv = *reinterpret_cast<const float4v *>(gp);
        }
        fp += J;
        gp += J;
        float ai[K];
#pragma unroll
        for (int k = 0; k < K; ++k) ai[k] = rd[r0 + r][k];
        const float ci = rd[r0 + r][K];
        float part[RP];
#pragma unroll
        for (int q = 0; q < RP; ++q) part[q] = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float g = dv[v] * fv[v];
            part[0] += g;
#pragma unroll
            for (int k = 0; k < K; ++k) part[1 + k] = fmaf(g, bj[v][k], part[1 + k]);
            part[K + 1] = fmaf(g, nb[v], part[K + 1]);
            float h = ci * g;
            tc[v] += h;
#pragma unroll
            for (int k = 0; k < K; ++k) Tc[v][k] = fmaf(h, ai[k], Tc[v][k]);
        }
#pragma unroll
        for (int q = 0; q < RP; ++q) part[q] = wave_sum(part[q]);
        if (lane == 0) {
#pragma unroll
            for (int q = 0; q < RP; ++q) rp[q] = part[q];
        }
        rp += RP;
    }

    // column partials: add the four waves in fixed order, one thread per column
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        cred[wave][0][lane * 4 + v] = tc[v];
#pragma unroll
        for (int k = 0; k < K; ++k) cred[wave][1 + k][lane * 4 + v] = Tc[v][k];
    }
    __syncthreads();
    const int j = blockIdx.x * BWD_TJ + tid;
    if (j < J) {
#pragma unroll
        for (int q = 0; q < CP; ++q) {
            float s = (cred[0][q][tid] + cred[1][q][tid]) + (cred[2][q][tid] + cred[3][q][tid]);
            colp[((size_t)blockIdx.y * CP + q) * J + j] = s;
        }
    }
}

// rows: da, dc diagonal, r_i
template <int K>
__global__ __launch_bounds__(256) void k_worked_finish_rows(const float *__restrict__ a, const float *__restrict__ c,
                                                            const float *__restrict__ rowp, int n_jt,
                                                            float *__restrict__ da, float *__restrict__ dc,
                                                            float *__restrict__ rsum, int I, int c_ld) {
    constexpr int RP = K + 2;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= I) return;
    double acc[RP];
#pragma unroll
    for (int q = 0; q < RP; ++q) acc[q] = 0.0;
    for (int jt = 0; jt < n_jt; ++jt) {
        const float *p = rowp + ((size_t)jt * I + i) * RP;
#pragma unroll
        for (int q = 0; q < RP; ++q) acc[q] += (double)p[q];
    }
    const double ci = (double)c[(size_t)i * c_ld + i];
    double na = 0.0, cross = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        double ak = (double)a[(size_t)i * K + k];
        na += ak * ak;
        cross += ak * acc[1 + k];
        if (da) da[(size_t)i * K + k] = (float)(-2.0 * ci * (ak * acc[0] + acc[1 + k]));
    }
    if (dc) dc[(size_t)i * c_ld + i] = (float)(-(na * acc[0] + 2.0 * cross + acc[K + 1]));
    rsum[i] = (float)acc[0];
}

// columns: db
template <int K>
__global__ __launch_bounds__(256) void k_worked_finish_cols(const float *__restrict__ b,
                                                            const float *__restrict__ colp, int n_it,
                                                            float *__restrict__ db, int J) {
    constexpr int CP = K + 1;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= J) return;
    double acc[CP];
#pragma unroll
    for (int q = 0; q < CP; ++q) acc[q] = 0.0;
    for (int it = 0; it < n_it; ++it)
#pragma unroll
        for (int q = 0; q < CP; ++q) acc[q] += (double)colp[((size_t)it * CP + q) * J + j];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        double bk = (double)b[(size_t)j * K + k];
        db[(size_t)j * K + k] = (float)(-2.0 * (acc[1 + k] + bk * acc[0]));
    }
}

// dd_m = -3 d_m^2 * sum over the window coordinate of r_i.  Masks and the window come from the plan of d:
// kernel coordinate `lvl_win` is the window, the other coordinate (the collapsed j) is already summed in r.
__global__ __launch_bounds__(256) void k_worked_dd(const GatherPlan P, int lvl_win, int iy, int iz,
                                                   const float *__restrict__ d, const float *__restrict__ rsum,
                                                   float *__restrict__ dd, int n) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= n) return;
    int32_t beta[kMaxRank] = {m, 0, 0, 0}, y[kMaxRank] = {0, 0, 0, 0}, z[kMaxKernel] = {0, 0, 0, 0};
    float out = 0.f;
    if (gather_prepare(P, beta, y)) {
        int32_t lo, hi;
        gather_bounds(P, lvl_win, y, z, lo, hi);
        double s = 0.0;
        for (int32_t w = lo; w <= hi; ++w) s += (double)rsum[iy * y[0] + iz * w];
        const double dm = (double)d[m];
        out = (float)(-3.0 * dm * dm * s);
    }
    dd[m] = out;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct WorkedWs {
    float *rowp, *colp, *rsum;
    int n_jt, n_it;
};

static WorkedWs carve(void *ws, int64_t I, int64_t J, int64_t K) {
    WorkedWs w;
    w.n_jt = (int)((J + BWD_TJ - 1) / BWD_TJ);
    w.n_it = (int)((I + BWD_TI - 1) / BWD_TI);
    char *p = static_cast<char *>(ws);
    w.rowp = reinterpret_cast<float *>(p);
    p += align256((size_t)w.n_jt * I * (K + 2) * 4);
    w.colp = reinterpret_cast<float *>(p);
    p += align256((size_t)w.n_it * (K + 1) * J * 4);
    w.rsum = reinterpret_cast<float *>(p);
    return w;
}

template <int K>
static int fwd_k(const tad_plan &pl, const void *const *args, void *f, hipStream_t s) {
    const int I = (int)pl.fast.I, J = (int)pl.fast.J;
    dim3 grid((J + 1023) / 1024, (I + FWD_TI - 1) / FWD_TI);
    TAD_LAUNCH("k_worked_forward", (k_worked_forward<K>), grid, dim3(256), 0, s, (const float *)args[0],
               (const float *)args[1], (const float *)args[2], (const float *)args[3], (float *)f, I, J,
               (int)pl.fast.c_ld);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

template <int K>
static int bwd_k(const tad_plan &pl, const void *const *args, const void *f, const void *df, void *const *dx,
                 void *ws, hipStream_t s) {
    const int I = (int)pl.fast.I, J = (int)pl.fast.J, c_ld = (int)pl.fast.c_ld;
    WorkedWs w = carve(ws, I, J, K);
    const float *a = (const float *)args[0], *b = (const float *)args[1], *c = (const float *)args[2],
                *d = (const float *)args[3];
    float *dc = (float *)dx[2];
    dim3 grid(w.n_jt, w.n_it);
    TAD_LAUNCH("k_worked_backward", (k_worked_backward<K>), grid, dim3(256), 0, s, a, b, c, (const float *)f,
               (const float *)df, dc, (long long)pl.arg_count[2], w.rowp, w.colp, I, J, c_ld);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dx[0] || dx[2] || dx[3]) {
        TAD_LAUNCH("k_worked_finish_rows", (k_worked_finish_rows<K>), dim3((I + 255) / 256), dim3(256), 0, s, a, c,
                   w.rowp, w.n_jt, (float *)dx[0], dc, w.rsum, I, c_ld);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    if (dx[1]) {
        TAD_LAUNCH("k_worked_finish_cols", (k_worked_finish_cols<K>), dim3((J + 255) / 256), dim3(256), 0, s, b,
                   w.colp, w.n_it, (float *)dx[1], J);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    if (dx[3]) {
        const int n = (int)pl.arg_count[3];
        TAD_LAUNCH("k_worked_dd", k_worked_dd, dim3((n + 255) / 256), dim3(256), 0, s, pl.ap[3].dev,
                   pl.fast.dd_level, pl.fast.dd_iy, pl.fast.dd_iz, d, w.rsum, (float *)dx[3], n);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

#define TAD_K_SWITCH(fn, ...)                       \
    switch (pl.fast.K) {                            \
    case 1: return fn<1>(__VA_ARGS__);              \
    case 2: return fn<2>(__VA_ARGS__);              \
    case 3: return fn<3>(__VA_ARGS__);              \
    case 4: return fn<4>(__VA_ARGS__);              \
    case 5: return fn<5>(__VA_ARGS__);              \
    case 6: return fn<6>(__VA_ARGS__);              \
    case 7: return fn<7>(__VA_ARGS__);              \
    case 8: return fn<8>(__VA_ARGS__);              \
    default: return TAD_EUNSUPPORTED;               \
    }

int worked_forward(const tad_plan &pl, const void *const *args, void *f, hipStream_t s) {
    TAD_K_SWITCH(fwd_k, pl, args, f, s)
}

int worked_backward(const tad_plan &pl, const void *const *args, const void *f, const void *df,
                    void *const *dx, void *ws, hipStream_t s) {
    TAD_K_SWITCH(bwd_k, pl, args, f, df, dx, ws, s)
}

}  // namespace tad
