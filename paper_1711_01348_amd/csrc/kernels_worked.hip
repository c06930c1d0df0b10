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

#include <algorithm>

#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "launch_geom.h"

namespace tad {

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

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
        __builtin_nontemporal_store(e, reinterpret_cast<float4v *>(fp));
        fp += J;
    }
}

// ---------------------------------------------------------------------------------------------
// backward main pass.  Block = 4 waves over the same BWD_TJ = 512 columns (lane owns columns
// 4*lane..4*lane+3 and 256+4*lane..+3), each wave a quarter of the block's BWD_TI rows, four rows per
// step.  Column sums stay in registers for the whole tile; row sums are reduced across the wave with
// DPP adds and written once per (row, column tile).
// ---------------------------------------------------------------------------------------------

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, ROW_MASK == 0xf);
    return v + __int_as_float(t);
}

// One step of the sum over the 64 lanes, applied to N independent values (consecutive instructions do not depend
// on each other, so the wait states a dependent DPP chain needs are filled with useful work).  After the six
// steps the total is valid in lane 63; the other lanes hold partial sums nobody reads.  The broadcast steps run
// on all rows (every step is then one fused add): row r receives lane 15 of row r - 1 and rows 2, 3 receive lane
// 31, which gives lane 63 = (t3 + t2) + (t1 + t0), the order the masked form has.
template <int STEP, int N>
__device__ __forceinline__ void wave_sum_step(float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        if (STEP == 0) v[i] = dpp_add<0x111, 0xf>(v[i]);        // row_shr:1
        else if (STEP == 1) v[i] = dpp_add<0x112, 0xf>(v[i]);   // row_shr:2
        else if (STEP == 2) v[i] = dpp_add<0x114, 0xf>(v[i]);   // row_shr:4
        else if (STEP == 3) v[i] = dpp_add<0x118, 0xf>(v[i]);   // row_shr:8 -> lane 15 of every row of 16 holds the row total
        else if (STEP == 4) v[i] = dpp_add<0x142, 0xf>(v[i]);   // row_bcast:15
        else v[i] = dpp_add<0x143, 0xf>(v[i]);                  // row_bcast:31
    }
}
template <int N>
__device__ __forceinline__ void wave_sum_lane63(float (&v)[N]) {
    wave_sum_step<0>(v); wave_sum_step<1>(v); wave_sum_step<2>(v);
    wave_sum_step<3>(v); wave_sum_step<4>(v); wave_sum_step<5>(v);
}

constexpr int BWD_RB = 4;   // rows per step

template <int K>
__global__ __launch_bounds__(256) void k_worked_backward(const float *__restrict__ a, const float *__restrict__ b,
                                                         const float *__restrict__ c, const float *__restrict__ f,
                                                         const float *__restrict__ df, float *__restrict__ rowp,
                                                         float *__restrict__ colp, int I, int J, int c_ld) {
    constexpr int RW = K + 1;      // c_ii a_i0..c_ii a_i{K-1}, c_ii
    constexpr int RP = K + 2;      // row partials: r, P_0..P_{K-1}, Q
    constexpr int CP = K + 1;      // column partials: t, T_0..T_{K-1}
    constexpr int WR = BWD_TI / 4; // rows per wave
    __shared__ float rd[BWD_TI][RW];
    __shared__ float rows_out[RP][BWD_TI];
    __shared__ float cred[4][CP][BWD_TJ];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = blockIdx.y * BWD_TI;
    const int jb = blockIdx.x * BWD_TJ;

    for (int t = tid; t < BWD_TI; t += 256) {
        const int i = i0 + t;
        float ci = 0.f;
        if (i < I) ci = c[(size_t)i * c_ld + i];
#pragma unroll
        for (int k = 0; k < K; ++k) rd[t][k] = i < I ? ci * a[(size_t)i * K + k] : 0.f;
        rd[t][K] = ci;
    }
    __syncthreads();

    int jc[2];
    bool live[2];
    float bj[2][4][K], nb[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        jc[h] = jb + h * 256 + lane * 4;
        live[h] = jc[h] < J;
        const float *bp = b + (size_t)(live[h] ? jc[h] : 0) * K;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            nb[h][v] = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float bv = bp[v * K + k];     // J % 4 == 0: a live lane owns four existing columns
                bj[h][v][k] = live[h] ? bv : 0.f;
                nb[h][v] = fmaf(bj[h][v][k], bj[h][v][k], nb[h][v]);
            }
        }
    }
    float tc[2][4], Tc[2][4][K];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            tc[h][v] = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) Tc[h][v][k] = 0.f;
        }

    const int r0 = wave * WR;
    const int rows = max(0, min(WR, I - (i0 + r0)));
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    const bool all_columns = jb + BWD_TJ <= J;   // the same for the whole block
    for (int rb = 0; rb < WR; rb += BWD_RB) {
        float part[BWD_RB * RP];
#pragma unroll
        for (int q = 0; q < BWD_RB * RP; ++q) part[q] = 0.f;
        if (rb < rows) {
            float4v fv[BWD_RB][2], dv[BWD_RB][2];
            if (all_columns && rb + BWD_RB <= rows) {
                // inside the tensor as a whole (the case of every step but those at the edges): plain loads
#pragma unroll
                for (int r = 0; r < BWD_RB; ++r)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const size_t off = (size_t)(i0 + r0 + rb + r) * J + jc[h];
                        fv[r][h] = __builtin_nontemporal_load(reinterpret_cast<const float4v *>(f + off));
                        dv[r][h] = __builtin_nontemporal_load(reinterpret_cast<const float4v *>(df + off));
                    }
            } else {
#pragma unroll
                for (int r = 0; r < BWD_RB; ++r)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const bool ok = live[h] && (rb + r) < rows;
                        const size_t off = (size_t)(i0 + r0 + rb + r) * J + jc[h];
                        fv[r][h] = ok ? *reinterpret_cast<const float4v *>(f + off) : zero4;
                        dv[r][h] = ok ? *reinterpret_cast<const float4v *>(df + off) : zero4;
                    }
            }
#pragma unroll
            for (int r = 0; r < BWD_RB; ++r) {
                float ai[K];
#pragma unroll
                for (int k = 0; k < K; ++k) ai[k] = rd[r0 + rb + r][k];
                const float ci = rd[r0 + rb + r][K];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float g = dv[r][h][v] * fv[r][h][v];
                        part[r * RP] += g;
#pragma unroll
                        for (int k = 0; k < K; ++k) part[r * RP + 1 + k] = fmaf(g, bj[h][v][k], part[r * RP + 1 + k]);
                        part[r * RP + K + 1] = fmaf(g, nb[h][v], part[r * RP + K + 1]);
                        tc[h][v] = fmaf(g, ci, tc[h][v]);
#pragma unroll
                        for (int k = 0; k < K; ++k) Tc[h][v][k] = fmaf(g, ai[k], Tc[h][v][k]);
                    }
            }
            wave_sum_lane63(part);
        }
        if (lane == 63) {
#pragma unroll
            for (int r = 0; r < BWD_RB; ++r)
#pragma unroll
                for (int q = 0; q < RP; ++q) rows_out[q][r0 + rb + r] = part[r * RP + q];
        }
    }

    // column partials: add the four waves in fixed order, one thread per column (two columns per thread)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            cred[wave][0][h * 256 + lane * 4 + v] = tc[h][v];
#pragma unroll
            for (int k = 0; k < K; ++k) cred[wave][1 + k][h * 256 + lane * 4 + v] = Tc[h][v][k];
        }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int col = h * 256 + tid, j = jb + col;
        if (j < J) {
#pragma unroll
            for (int q = 0; q < CP; ++q) {
                float s = (cred[0][q][col] + cred[1][q][col]) + (cred[2][q][col] + cred[3][q][col]);
                colp[((size_t)blockIdx.y * CP + q) * J + j] = s;
            }
        }
    }
    // row partials of the tile, rowp[jt][q][i], contiguous in i
    for (int t = tid; t < BWD_TI; t += 256) {
        const int i = i0 + t;
        if (i < I) {
#pragma unroll
            for (int q = 0; q < RP; ++q) rowp[((size_t)blockIdx.x * RP + q) * I + i] = rows_out[q][t];
        }
    }
}

// Dense zero fill of a gradient whose non-zero elements are written afterwards (cokernel mask: only the
// diagonal of dc is non-zero).  A pure write stream runs faster than the same stores mixed into a read pass.
constexpr int FILL_U = 1;   // 16-byte stores per thread
__global__ __launch_bounds__(256) void k_fill_zero(float *__restrict__ p, long long n) {
    // every block writes one contiguous 4 KiB piece: 41 us for 256 MiB against 45 / 47 us with 8 / 16 KiB pieces and
    // more with grid-stride or tiled fills
    const long long n4 = n >> 2;
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    const long long lo = (long long)blockIdx.x * (256 * FILL_U) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < FILL_U; ++u) {
        const long long q = lo + 256 * u;
        if (q < n4) __builtin_nontemporal_store(z, reinterpret_cast<float4v *>(p) + q);
    }
    if (blockIdx.x == 0 && threadIdx.x < (int)(n & 3)) p[(n4 << 2) + threadIdx.x] = 0.f;
}

// Finishing pass, one launch with three block roles, 64 outputs per block; the four waves of a block split
// the tile partials (wave w takes tiles w, w+4, ...) and are combined in fixed order through LDS.
//   rows:  da, diagonal of dc               (sum of the row partials over the column tiles)
//   cols:  db                               (sum of the column partials over the row tiles)
//   dd:    dd_m = -3 d_m^2 * sum over the window coordinate of r_i; masks and the window come from the
//          plan of d (loop-free copy of its rows): one kernel coordinate is the window, the other one (j)
//          is already summed in the row partials.
template <int K>
__global__ __launch_bounds__(256) void k_worked_finish(const FlatFeas feas, const FlatLevel win, int iy, int iz,
                                                       const float *__restrict__ a, const float *__restrict__ b,
                                                       const float *__restrict__ c, const float *__restrict__ d,
                                                       const float *__restrict__ rowp, int n_jt,
                                                       const float *__restrict__ colp, int n_it,
                                                       float *__restrict__ da, float *__restrict__ db,
                                                       float *__restrict__ dc, float *__restrict__ dd, int I,
                                                       int J, int c_ld, int n_d, int blocks_rows, int blocks_cols) {
    constexpr int RP = K + 2, CP = K + 1;
    __shared__ double red[4][RP][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int blk = blockIdx.x;
    if (blk < blocks_rows) {
        const int i = blk * 64 + lane;
        double acc[RP];
#pragma unroll
        for (int q = 0; q < RP; ++q) acc[q] = 0.0;
        if (i < I)
            for (int jt = wave; jt < n_jt; jt += 4)
#pragma unroll
                for (int q = 0; q < RP; ++q) acc[q] += (double)rowp[((size_t)jt * RP + q) * I + i];
#pragma unroll
        for (int q = 0; q < RP; ++q) red[wave][q][lane] = acc[q];
        __syncthreads();
        if (wave != 0 || i >= I) return;
#pragma unroll
        for (int q = 0; q < RP; ++q) acc[q] = (red[0][q][lane] + red[1][q][lane]) + (red[2][q][lane] + red[3][q][lane]);
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
        return;
    }
    blk -= blocks_rows;
    if (blk < blocks_cols) {
        const int j = blk * 64 + lane;
        double acc[CP];
#pragma unroll
        for (int q = 0; q < CP; ++q) acc[q] = 0.0;
        if (j < J && db)
            for (int it = wave; it < n_it; it += 4)
#pragma unroll
                for (int q = 0; q < CP; ++q) acc[q] += (double)colp[((size_t)it * CP + q) * J + j];
#pragma unroll
        for (int q = 0; q < CP; ++q) red[wave][q][lane] = acc[q];
        __syncthreads();
        if (wave != 0 || j >= J || !db) return;
#pragma unroll
        for (int q = 0; q < CP; ++q) acc[q] = (red[0][q][lane] + red[1][q][lane]) + (red[2][q][lane] + red[3][q][lane]);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            // the column partials carry c_ii a_ik and c_ii already:  db_jk = -2 (T_jk + b_jk t_j)
            double bk = (double)b[(size_t)j * K + k];
            db[(size_t)j * K + k] = (float)(-2.0 * (acc[1 + k] + bk * acc[0]));
        }
        return;
    }
    blk -= blocks_cols;
    const int m = blk * 64 + lane;
    double s = 0.0;
    bool nonzero = false;
    if (m < n_d && dd) {
        const int32_t y[3] = {m, 0, 0};   // the transformed index is the gradient index (checked on the host)
        if (flat_feasible(feas, y)) {
            nonzero = true;
            int32_t lo, hi;
            flat_bounds(win, y, lo, hi);
            for (int32_t w = lo; w <= hi; ++w) {
                const int i = iy * y[0] + iz * w;
                for (int jt = wave; jt < n_jt; jt += 4) s += (double)rowp[((size_t)jt * RP) * I + i];
            }
        }
    }
    red[wave][0][lane] = s;
    __syncthreads();
    if (wave != 0 || m >= n_d || !dd) return;
    float out = 0.f;
    if (nonzero) {
        s = (red[0][0][lane] + red[1][0][lane]) + (red[2][0][lane] + red[3][0][lane]);
        const double dm = (double)d[m];
        out = (float)(-3.0 * dm * dm * s);
    }
    dd[m] = out;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct WorkedWs {
    float *rowp, *colp;
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
               (const float *)df, w.rowp, w.colp, I, J, c_ld);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dc) {
        // after the read pass: a write burst right before it slows the reads down
        const long long n = pl.arg_count[2];
        const int g = (int)((n / 4 + 256 * FILL_U - 1) / (256 * FILL_U) + 1);
        TAD_LAUNCH("k_fill_zero", k_fill_zero, dim3(g), dim3(256), 0, s, dc, n);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    {
        const int n_d = (int)pl.arg_count[3];
        const int br = (I + 63) / 64, bc = (J + 63) / 64, bd = (n_d + 63) / 64;
        TAD_LAUNCH("k_worked_finish", (k_worked_finish<K>), dim3(br + bc + bd), dim3(256), 0, s, pl.fast.feas,
                   pl.fast.flat[0], pl.fast.dd_iy, pl.fast.dd_iz, a, b, c, d, w.rowp, w.n_jt, w.colp, w.n_it,
                   (float *)dx[0], (float *)dx[1], dc, (float *)dx[3], I, J, c_ld, n_d, br, bc);
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
