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
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const float4v *>(row + j + u * 1024));
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
constexpr int AD_FTI = 2;     // rows per forward block (small tiles for a pure write stream: 11.2 us against 11.8 with 32 rows)

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

// Backward, first pass.  A block takes one aligned tile of df (AD_TR rows x AD_TC columns, 16-byte loads along the
// rows) and sums it along its antidiagonals: element (r, c) of the tile belongs to the sum with offset r + c.  Each of
// its four waves takes 64 rows.  A lane loads four consecutive columns, so over four rows it meets the offsets
// 4 lane .. 4 lane + 6: its own group of four sums and three sums of the next group.  The groups sit in a ring over
// the lanes that moves down by one lane every four rows (wave_shl:1), so the group a lane holds stays the one its
// next four rows start at; the carry for the next group is added while it moves in.  The group that leaves lane 0 is
// finished.  The waves' sums are combined in LDS in a fixed order and the block writes 4 (64 + AD_TR / 4) sums per
// tile; nothing here needs the plan: the window of Sec. 1's dx_k = sum_i df_{i,k-i} restricted to a tile is the tile's
// whole antidiagonal, and the finishing pass takes the tiles that the plan's window meets.
constexpr int AD_TR = AD_TILE_ROWS, AD_TC = AD_TILE_COLS, AD_WAVES = 4;
constexpr int AD_WR = AD_TR / AD_WAVES;          // rows per wave
constexpr int AD_G = AD_WR / 4;                  // groups of four rows per wave
constexpr int AD_NB = 64 + AD_G;                 // groups of four sums per wave
constexpr int AD_OUTB = 64 + AD_G * AD_WAVES;    // ... per tile
static_assert(AD_TC == 256 && AD_G % 2 == 0 && AD_OUTB * 4 == AD_TILE_SUMS, "tile geometry");

__device__ __forceinline__ float lane_above(float v) {   // value of lane + 1; 0 in lane 63
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, true));
}

template <bool FULL>
__device__ __forceinline__ void antidiag_tile(const float *__restrict__ df, float4v (*outb)[AD_NB], int I, int J, int i0,
                                              int col, int lane, int wave) {
    const float *p = df + (size_t)i0 * J + col;
    float4v A = {0.f, 0.f, 0.f, 0.f};
    const bool col_ok = FULL || col < J;
    for (int g = 0; g < AD_G; g += 2) {
        float4v v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (FULL || (col_ok && i0 + g * 4 + r < I))   // read once: non-temporal (12.0 us against 12.7 alone)
                v[r] = __builtin_nontemporal_load(reinterpret_cast<const float4v *>(p + (size_t)r * J));
            else v[r] = float4v{0.f, 0.f, 0.f, 0.f};
        }
        p += (size_t)8 * J;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4v v0 = v[4 * h], v1 = v[4 * h + 1], v2 = v[4 * h + 2], v3 = v[4 * h + 3];
            A[0] += v0[0];
            A[1] += v0[1] + v1[0];
            A[2] += (v0[2] + v1[1]) + v2[0];
            A[3] += (v0[3] + v1[2]) + (v2[1] + v3[0]);
            const float c0 = (v1[3] + v2[2]) + v3[1], c1 = v2[3] + v3[2], c2 = v3[3];
            if (lane == 0) outb[wave][g + h] = A;
            A[0] = lane_above(A[0]) + c0;
            A[1] = lane_above(A[1]) + c1;
            A[2] = lane_above(A[2]) + c2;
            A[3] = lane_above(A[3]);
        }
    }
    outb[wave][AD_G + lane] = A;
}

__global__ __launch_bounds__(64 * AD_WAVES) void k_antidiag_backward(const float *__restrict__ df, float *__restrict__ part,
                                                                     int I, int J, int n_ct) {
    __shared__ float4v outb[AD_WAVES][AD_NB];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x, t = blockIdx.y;
    const int i0 = t * AD_TR + wave * AD_WR, col = c * AD_TC + lane * 4;
    if ((t + 1) * AD_TR <= I && (c + 1) * AD_TC <= J) antidiag_tile<true>(df, outb, I, J, i0, col, lane, wave);
    else antidiag_tile<false>(df, outb, I, J, i0, col, lane, wave);
    __syncthreads();
    float4v *out = reinterpret_cast<float4v *>(part + (size_t)(t * n_ct + c) * AD_TILE_SUMS);
    for (int b = threadIdx.x; b < AD_OUTB; b += 64 * AD_WAVES) {
        float4v s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < AD_WAVES; ++w) {
            const int q = b - AD_G * w;      // wave w starts AD_WR rows, i.e. AD_G groups, further down
            if (q >= 0 && q < AD_NB) s += outb[w][q];
        }
        out[b] = s;
    }
}

// Second pass: dx_m = phi'(x_m) * sum over the tiles that the plan's window of m meets.  The window (Sec. 5.1 range
// rows, kernel coordinate z with i = iy*y + iz*z, iz = +-1) gives the rows of df that carry terms of m; a tile row t
// holds the sum with offset m - AD_TR t of two neighbouring tile columns.  A block finishes 16 elements: thread
// (e, q) takes element e and the tile rows q, q + 16, ... of its window, so that every thread has one short round of
// independent loads; the 16 partial sums of an element are added in fp64 in a fixed order.
constexpr int AD_FIN_M = 16, AD_FIN_Q = 16;
template <int BODY>
__global__ __launch_bounds__(AD_FIN_M * AD_FIN_Q) void k_antidiag_finish(const FlatFeas feas, const FlatLevel win, int iy, int iz,
                                                                         const float *__restrict__ x,
                                                                         const float *__restrict__ part, int n_ct,
                                                                         float *__restrict__ dx, int n_x) {
    __shared__ double red[AD_FIN_Q][AD_FIN_M];
    const int e = threadIdx.x % AD_FIN_M, q = threadIdx.x / AD_FIN_M;
    const int m = blockIdx.x * AD_FIN_M + e;
    double s = 0.0;
    float xm = 0.f;
    if (q == 0 && m < n_x) xm = x[m];   // issued with the loads of the partial sums, not after the barrier
    if (m < n_x) {
        const int32_t y[3] = {m, 0, 0};   // the transformed index is the gradient index (checked on the host)
        int32_t lo = 0, hi = -1;
        if (flat_feasible(feas, y)) flat_bounds(win, y, lo, hi);
        if (lo <= hi) {
            const int ia = iy * m + iz * lo, ib = iy * m + iz * hi;
            const int t_lo = min(ia, ib) / AD_TR, t_hi = max(ia, ib) / AD_TR;
            for (int t = t_lo + q; t <= t_hi; t += AD_FIN_Q) {
                const int off = m - t * AD_TR;                 // >= 0: the window's rows do not exceed m
                if (off < 0) continue;
                const int c1 = off / AD_TC, o = off % AD_TC;
                float a = 0.f, b = 0.f;
                if (c1 < n_ct) a = part[(size_t)(t * n_ct + c1) * AD_TILE_SUMS + o];
                if (c1 >= 1 && c1 - 1 < n_ct && o + AD_TC < AD_TILE_SUMS) b = part[(size_t)(t * n_ct + c1 - 1) * AD_TILE_SUMS + o + AD_TC];
                s += (double)a + (double)b;
            }
        }
    }
    red[q][e] = s;
    __syncthreads();
    if (q == 0 && m < n_x) {
        s = 0.0;
#pragma unroll
        for (int w = 0; w < AD_FIN_Q; ++w) s += red[w][e];
        dx[m] = (float)((double)dphi<BODY>(xm) * s);
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
        const int n_rt = (I + AD_TR - 1) / AD_TR, n_ct = (J + AD_TC - 1) / AD_TC;
        float *part = (float *)ws;
        // the kernels address f as i * J + j with j = m - i: only the plain sum of the two function indices
        if (pl.fast.dd_iy + pl.fast.jy != 1 || pl.fast.dd_iz + pl.fast.jz != 0) return TAD_EUNSUPPORTED;
        TAD_LAUNCH("k_antidiag_backward", k_antidiag_backward, dim3(n_ct, n_rt), dim3(64 * AD_WAVES), 0, s, df, part, I, J,
                   n_ct);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
        TAD_UNARY_SWITCH(pl.expr.body, TAD_LAUNCH("k_antidiag_finish", (k_antidiag_finish<B_>),
                                                  dim3((n_x + AD_FIN_M - 1) / AD_FIN_M), dim3(AD_FIN_M * AD_FIN_Q), 0, s, pl.fast.feas,
                                                  pl.fast.flat[0], pl.fast.dd_iy, pl.fast.dd_iz, x, part, n_ct, dx, n_x));
        break;
    }
    default: return TAD_EUNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

}  // namespace tad
