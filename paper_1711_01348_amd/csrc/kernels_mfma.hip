// Worked expression with a long summed index (K a multiple of 32, fp32): the contraction over k is a
// genuine dense matrix product, so it runs on the matrix cores (v_mfma_f32_32x32x2f32).
//
//   forward   s_ij = |a_i|^2 + |b_j|^2 + 2 a_i . b_j        (expanded square; a . b^T on MFMA)
//             f_ij = exp(-(c_ii s_ij + D_i)),  D_i = sum_k d_{i+k}^3
//   backward  G_ij = df_ij f_ij
//             P = G b        (I x K, contraction over the collapsed kernel coordinate j, split in chunks)
//             T = (c G)^T a  (J x K, contraction over the collapsed kernel coordinate i, split in chunks)
//             r_i = sum_j G_ij, Q_i = sum_j G_ij |b_j|^2, t_j = sum_i c_ii G_ij   (accumulated while G is staged)
//             da_ik = -2 c_ii (a_ik r_i + P_ik)      db_jk = -2 (T_jk + b_jk t_j)
//             dc_ii = -(|a_i|^2 r_i + 2 sum_k a_ik P_ik + Q_i)      dd_m = -3 d_m^2 sum_{i in window(m)} r_i
// All partial results are combined in a fixed order (no atomics).
//
// MFMA operand layout used below (wave64): A operand lane l = A[m = l % 32][k = l / 32],
// B operand lane l = B[k = l / 32][n = l % 32], result register r of lane l = D[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].
#include <hip/hip_runtime.h>

#include <algorithm>

#include "launch.h"
#include "plan_dev.h"
#include "profile.h"
#include "launch_geom.h"

namespace tad {

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr float kLog2eM = 1.4426950408889634f;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_m(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, ROW_MASK == 0xf);
    return v + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum63m(float v) {   // total valid in lane 63
    v = dpp_add_m<0x111, 0xf>(v);
    v = dpp_add_m<0x112, 0xf>(v);
    v = dpp_add_m<0x114, 0xf>(v);
    v = dpp_add_m<0x118, 0xf>(v);
    v = dpp_add_m<0x142, 0xa>(v);
    v = dpp_add_m<0x143, 0xc>(v);
    return v;
}

__device__ __forceinline__ void zero_acc(float16v (&acc)[2][2]) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
}

__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// ---------------------------------------------------------------------------------------------
// per-row and per-column quantities: rowv[i] = {|a_i|^2, -log2e c_ii, -log2e D_i, c_ii}, nb[j] = |b_j|^2
// one wave per row
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mfma_prep(const float *__restrict__ a, const float *__restrict__ b,
                                                   const float *__restrict__ c, const float *__restrict__ d,
                                                   float *__restrict__ rowv, float *__restrict__ nb, int I, int J,
                                                   int K, int c_ld) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row < I) {
        float na = 0.f, D = 0.f;
        for (int k = lane; k < K; k += 64) {
            const float av = a[(size_t)row * K + k], dv = d[row + k];
            na = fmaf(av, av, na);
            D = fmaf(dv * dv, dv, D);
        }
        na = wave_sum63m(na);
        D = wave_sum63m(D);
        if (lane == 63) {
            const float cv = c[(size_t)row * c_ld + row];
            rowv[row * 4 + 0] = na;
            rowv[row * 4 + 1] = -kLog2eM * cv;
            rowv[row * 4 + 2] = -kLog2eM * D;
            rowv[row * 4 + 3] = cv;
        }
    } else if (row - I < J) {
        const int j = row - I;
        float s = 0.f;
        for (int k = lane; k < K; k += 64) {
            const float bv = b[(size_t)j * K + k];
            s = fmaf(bv, bv, s);
        }
        s = wave_sum63m(s);
        if (lane == 63) nb[j] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// forward: block tile 128 x 128, 2 x 2 waves of 64 x 64, k tile 32, global -> register -> LDS staging
// ---------------------------------------------------------------------------------------------
constexpr int MF_KT = 32;
constexpr int MF_LD = 33;   // odd row stride: conflict-free ds_read_b32 of [row][k] tiles

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_mfma_forward(const float *__restrict__ a, const float *__restrict__ b,
                                                      const float *__restrict__ rowv, const float *__restrict__ nb,
                                                      float *__restrict__ f, int I, int J, int K) {
    __shared__ float smem[2 * 128 * MF_LD];   // A tile then B tile; reused as the output stage in the epilogue
    __shared__ float rv[128][4];
    float (*As)[MF_LD] = reinterpret_cast<float (*)[MF_LD]>(smem);
    float (*Bs)[MF_LD] = reinterpret_cast<float (*)[MF_LD]>(smem + 128 * MF_LD);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * 128, j0 = blockIdx.x * 128;
    if (tid < 128) {
        const int i = i0 + tid;
#pragma unroll
        for (int q = 0; q < 4; ++q) rv[tid][q] = i < I ? rowv[i * 4 + q] : 0.f;
    }
    float16v acc[2][2];
    zero_acc(acc);
    float4v ra[4], rb[4];
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    auto gload = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int idx = tid + 256 * p, row = idx >> 3, kq = idx & 7;
            ra[p] = (i0 + row < I) ? *reinterpret_cast<const float4v *>(a + (size_t)(i0 + row) * K + k0 + 4 * kq) : zero4;
            rb[p] = (j0 + row < J) ? *reinterpret_cast<const float4v *>(b + (size_t)(j0 + row) * K + k0 + 4 * kq) : zero4;
        }
    };
    gload(0);
    const int mrow = lane & 31, kof = lane >> 5;
    for (int k0 = 0; k0 < K; k0 += MF_KT) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int idx = tid + 256 * p, row = idx >> 3, kq = idx & 7;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                As[row][4 * kq + q] = ra[p][q];
                Bs[row][4 * kq + q] = rb[p][q];
            }
        }
        __syncthreads();
        if (k0 + MF_KT < K) gload(k0 + MF_KT);
        // the operands of step ks + 1 are read from LDS before the MFMAs of step ks are issued
        float a0 = As[wm * 64 + mrow][kof], a1 = As[wm * 64 + 32 + mrow][kof];
        float b0 = Bs[wn * 64 + mrow][kof], b1 = Bs[wn * 64 + 32 + mrow][kof];
#pragma unroll
        for (int ks = 0; ks < MF_KT / 2; ++ks) {
            float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
            if (ks + 1 < MF_KT / 2) {
                na0 = As[wm * 64 + mrow][2 * ks + 2 + kof];
                na1 = As[wm * 64 + 32 + mrow][2 * ks + 2 + kof];
                nb0 = Bs[wn * 64 + mrow][2 * ks + 2 + kof];
                nb1 = Bs[wn * 64 + 32 + mrow][2 * ks + 2 + kof];
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
        }
        __syncthreads();
    }
    // epilogue: f = exp2(c' (|a|^2 + |b|^2 + 2 a.b) + D').  Each wave stages 32 x 64 results at a time in its own
    // quarter of the tile memory (32 rows of 66 floats) and writes them as 16-byte stores, 256 bytes per row.
    // (the last barrier of the loop guarantees that nobody still reads the tiles)
    float *stage = smem + wave * (32 * 66);
    constexpr int kStageOk = (4 * 32 * 66 <= 2 * 128 * MF_LD) ? 1 : -1;
    static_assert(kStageOk == 1, "output stage does not fit in the tile memory");
#pragma unroll
    for (int tm = 0; tm < 2; ++tm) {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int j = j0 + wn * 64 + tn * 32 + mrow;
            const float nbj = j < J ? nb[j] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int mloc = acc_row(r, lane), m = wm * 64 + tm * 32 + mloc;
                const float s = rv[m][0] + nbj + 2.f * acc[tm][tn][r];
                stage[mloc * 66 + tn * 32 + mrow] = __builtin_amdgcn_exp2f(fmaf(rv[m][1], s, rv[m][2]));
            }
        }
        // the wave reads back only what it wrote itself: no barrier needed, LDS operations of a wave are ordered
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int rl = it * 4 + (lane >> 4), c = (lane & 15) * 4;
            const int i = i0 + wm * 64 + tm * 32 + rl, j = j0 + wn * 64 + c;
            if (i < I && j < J) {   // J % 4 == 0: the four columns exist together
                const float4v v = {stage[rl * 66 + c], stage[rl * 66 + c + 1], stage[rl * 66 + c + 2],
                                   stage[rl * 66 + c + 3]};
                *reinterpret_cast<float4v *>(f + (size_t)i * J + j) = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// backward contractions.  Block tile 64 (M) x 256 (N = k), 1 x 4 waves of 64 x 64, contraction tile 32.
//   TRANS_A = false:  M = i, contraction over j in [cs, ce):  A[m][kk] = df f            B[kk][n] = b[j][k]
//   TRANS_A = true:   M = j, contraction over i in [cs, ce):  A[m][kk] = c_ii df f (read transposed), B[kk][n] = a[i][k]
// out[(split * Mtot + m) * K + n]
// ---------------------------------------------------------------------------------------------
// While G is staged, the same thread keeps meeting the same rows (TRANS_A = false) or the same columns
// (TRANS_A = true), so the plain sums over the collapsed index are accumulated on the side:
//   TRANS_A = false:  sums[(split * 2 + 0) * I + i] = sum_j G_ij,  sums[(split * 2 + 1) * I + i] = sum_j G_ij |b_j|^2
//   TRANS_A = true:   sums[split * J + j] = sum_i c_ii G_ij
template <bool TRANS_A>
__global__ __launch_bounds__(256) void k_mfma_backward(const float *__restrict__ f, const float *__restrict__ df,
                                                       const float *__restrict__ bmat, const float *__restrict__ rowv,
                                                       const float *__restrict__ nb, float *__restrict__ out,
                                                       float *__restrict__ sums, int I, int J, int K, int chunk) {
    __shared__ float As[TRANS_A ? 32 : 64][TRANS_A ? 64 : MF_LD];
    __shared__ float Bs[32][256];
    __shared__ float tred[4][64];
    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const int Mtot = TRANS_A ? J : I, Ctot = TRANS_A ? I : J;
    const int m0 = blockIdx.x * 64, split = blockIdx.y, n0 = blockIdx.z * 256;
    const int cs = split * chunk, ce = min(Ctot, cs + chunk);
    float16v acc[2][2];
    zero_acc(acc);
    float4v ga[2], gb[8];
    // what the loads of G bring in; the products and the sums on the side are formed one tile later, when the
    // tile is staged, so that nothing waits for these loads before the matrix instructions of the current tile
    float4v rdf[2], rf[2], rnv[2];
    float rc[2];
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    float sr[2] = {0.f, 0.f}, sq[2] = {0.f, 0.f};   // TRANS_A = false: row sums of the thread's two rows
    float4v st = zero4;                               // TRANS_A = true: column sums of the thread's four columns
    auto gload = [&](int c0) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int idx = tid + 256 * p;
            rdf[p] = zero4; rf[p] = zero4; rnv[p] = zero4; rc[p] = 0.f;
            if (!TRANS_A) {
                const int row = idx >> 3, q = idx & 7;            // i = m0 + row, j = c0 + 4 q
                const int i = m0 + row, j = c0 + 4 * q;
                if (i < I && j < ce) {
                    const size_t off = (size_t)i * J + j;
                    rdf[p] = *reinterpret_cast<const float4v *>(df + off);
                    rf[p] = *reinterpret_cast<const float4v *>(f + off);
                    rnv[p] = *reinterpret_cast<const float4v *>(nb + j);
                }
            } else {
                const int kk = idx >> 4, q = idx & 15;            // i = c0 + kk, j = m0 + 4 q
                const int i = c0 + kk, j = m0 + 4 * q;
                if (i < ce && j < J) {
                    const size_t off = (size_t)i * J + j;
                    rdf[p] = *reinterpret_cast<const float4v *>(df + off);
                    rf[p] = *reinterpret_cast<const float4v *>(f + off);
                    rc[p] = rowv[i * 4 + 3];
                }
            }
        }
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int idx = tid + 256 * p, kk = idx >> 6, q = idx & 63;
            const int cc = c0 + kk, n = n0 + 4 * q;
            gb[p] = (cc < ce && n < K) ? *reinterpret_cast<const float4v *>(bmat + (size_t)cc * K + n) : zero4;
        }
    };
    auto gprep = [&]() {   // G of the loaded tile and its plain sums (zeros where nothing was loaded)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if (!TRANS_A) {
                ga[p] = rdf[p] * rf[p];
                sr[p] += (ga[p][0] + ga[p][1]) + (ga[p][2] + ga[p][3]);
                sq[p] += (ga[p][0] * rnv[p][0] + ga[p][1] * rnv[p][1]) + (ga[p][2] * rnv[p][2] + ga[p][3] * rnv[p][3]);
            } else {
                ga[p] = rdf[p] * rf[p] * rc[p];
                st += ga[p];
            }
        }
    };
    gload(cs);
    const int mrow = lane & 31, kof = lane >> 5;
    for (int c0 = cs; c0 < ce; c0 += MF_KT) {
        gprep();
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int idx = tid + 256 * p;
            if (!TRANS_A) {
                const int row = idx >> 3, q = idx & 7;
#pragma unroll
                for (int e = 0; e < 4; ++e) As[row][4 * q + e] = ga[p][e];
            } else {
                const int kk = idx >> 4, q = idx & 15;
                *reinterpret_cast<float4v *>(&As[kk][4 * q]) = ga[p];
            }
        }
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int idx = tid + 256 * p, kk = idx >> 6, q = idx & 63;
            *reinterpret_cast<float4v *>(&Bs[kk][4 * q]) = gb[p];
        }
        __syncthreads();
        if (c0 + MF_KT < ce) gload(c0 + MF_KT);
        auto afrag = [&](int kk, int half) -> float {
            return TRANS_A ? As[kk + kof][32 * half + mrow] : As[32 * half + mrow][kk + kof];
        };
        // the operands of step ks + 1 are read from LDS before the MFMAs of step ks are issued
        float a0 = afrag(0, 0), a1 = afrag(0, 1);
        float b0 = Bs[kof][wn * 64 + mrow], b1 = Bs[kof][wn * 64 + 32 + mrow];
#pragma unroll
        for (int ks = 0; ks < MF_KT / 2; ++ks) {
            float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
            if (ks + 1 < MF_KT / 2) {
                na0 = afrag(2 * ks + 2, 0);
                na1 = afrag(2 * ks + 2, 1);
                nb0 = Bs[2 * ks + 2 + kof][wn * 64 + mrow];
                nb1 = Bs[2 * ks + 2 + kof][wn * 64 + 32 + mrow];
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
        }
        __syncthreads();
    }
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
        const int n = n0 + wn * 64 + tn * 32 + mrow;
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + tm * 32 + acc_row(r, lane);
                if (m < Mtot && n < K) out[((size_t)split * Mtot + m) * K + n] = acc[tm][tn][r];
            }
    }
    if (blockIdx.z != 0) return;
    if (!TRANS_A) {
        // eight consecutive lanes share a row: add them in a fixed order
#pragma unroll
        for (int p = 0; p < 2; ++p) {
#pragma unroll
            for (int m = 1; m <= 4; m <<= 1) {
                sr[p] += __shfl_xor(sr[p], m, 64);
                sq[p] += __shfl_xor(sq[p], m, 64);
            }
            const int i = m0 + (tid >> 3) + 32 * p;
            if ((tid & 7) == 0 && i < I) {
                sums[((size_t)split * 2 + 0) * I + i] = sr[p];
                sums[((size_t)split * 2 + 1) * I + i] = sq[p];
            }
        }
    } else {
        // lanes q, q+16, q+32, q+48 of every wave hold the same four columns: add within the wave, then the waves
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            st[e] += __shfl_xor(st[e], 16, 64);
            st[e] += __shfl_xor(st[e], 32, 64);
        }
        if (lane < 16)
#pragma unroll
            for (int e = 0; e < 4; ++e) tred[wn][lane * 4 + e] = st[e];
        __syncthreads();
        if (tid < 64) {
            const int j = m0 + tid;
            if (j < J) sums[(size_t)split * J + j] = (tred[0][tid] + tred[1][tid]) + (tred[2][tid] + tred[3][tid]);
        }
    }
}

__global__ __launch_bounds__(256) void k_mfma_fill_zero(float *__restrict__ p, long long n) {
    const long long n4 = n >> 2;
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    const long long stride = (long long)gridDim.x * 256;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < n4; q += stride)
        reinterpret_cast<float4v *>(p)[q] = z;
    if (blockIdx.x == 0 && threadIdx.x < (int)(n & 3)) p[(n4 << 2) + threadIdx.x] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// finishing: one wave per output row, lane owns four consecutive k.
// Blocks [0, blocks_rows): rows i (da, dc_ii, r_i); the rest: rows j (db).  Fixed summation order.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mfma_finish(const float *__restrict__ a, const float *__restrict__ b,
                                                     const float *__restrict__ rowv, const float *__restrict__ Ppart,
                                                     const float *__restrict__ Tpart, int n_split,
                                                     const float *__restrict__ rowp, const float *__restrict__ colp,
                                                     float *__restrict__ da, float *__restrict__ db,
                                                     float *__restrict__ dc, float *__restrict__ rsum, int I, int J,
                                                     int K, int c_ld, int blocks_rows) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if ((int)blockIdx.x < blocks_rows) {
        const int i = blockIdx.x * 4 + wv;
        if (i >= I) return;
        double r = 0.0, Q = 0.0;
        for (int s = 0; s < n_split; ++s) {
            r += (double)rowp[((size_t)s * 2 + 0) * I + i];
            Q += (double)rowp[((size_t)s * 2 + 1) * I + i];
        }
        const double ci = (double)rowv[i * 4 + 3], na = (double)rowv[i * 4 + 0];
        float cross = 0.f;
        if (da || dc)
            for (int k = lane * 4; k < K; k += 256) {
                float4v P = {0.f, 0.f, 0.f, 0.f};
                for (int s = 0; s < n_split; ++s)
                    P += *reinterpret_cast<const float4v *>(Ppart + ((size_t)s * I + i) * K + k);
                const float4v av = *reinterpret_cast<const float4v *>(a + (size_t)i * K + k);
                if (da) {
                    float4v o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (float)(-2.0 * ci * ((double)av[e] * r + (double)P[e]));
                    *reinterpret_cast<float4v *>(da + (size_t)i * K + k) = o;
                }
                cross += (av[0] * P[0] + av[1] * P[1]) + (av[2] * P[2] + av[3] * P[3]);
            }
        cross = wave_sum63m(cross);
        if (lane == 63) {
            if (dc) dc[(size_t)i * c_ld + i] = (float)(-(na * r + 2.0 * (double)cross + Q));
            rsum[i] = (float)r;
        }
        return;
    }
    const int j = ((int)blockIdx.x - blocks_rows) * 4 + wv;
    if (j >= J || !db) return;
    double t = 0.0;
    for (int s = 0; s < n_split; ++s) t += (double)colp[(size_t)s * J + j];
    for (int k = lane * 4; k < K; k += 256) {
        float4v T = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < n_split; ++s) T += *reinterpret_cast<const float4v *>(Tpart + ((size_t)s * J + j) * K + k);
        const float4v bv = *reinterpret_cast<const float4v *>(b + (size_t)j * K + k);
        float4v o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (float)(-2.0 * ((double)T[e] + (double)bv[e] * t));
        *reinterpret_cast<float4v *>(db + (size_t)j * K + k) = o;
    }
}

// dd_m = -3 d_m^2 sum_{i in window(m)} r_i, one wave per m; window and masks from the plan of d
__global__ __launch_bounds__(256) void k_mfma_dd(const FlatFeas feas, const FlatLevel win, int iy, int iz,
                                                 const float *__restrict__ d, const float *__restrict__ rsum,
                                                 float *__restrict__ dd, int n_d) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= n_d) return;
    const int32_t y[3] = {m, 0, 0};
    float s = 0.f;
    const bool ok = flat_feasible(feas, y);
    if (ok) {
        int32_t lo, hi;
        flat_bounds(win, y, lo, hi);
        for (int32_t w = lo + lane; w <= hi; w += 64) s += rsum[iy * y[0] + iz * w];
    }
    s = wave_sum63m(s);
    if (lane == 63) {
        const float dm = d[m];
        dd[m] = ok ? -3.f * dm * dm * s : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct MfmaWs {
    float *rowv, *nb, *Ppart, *Tpart, *rowp, *colp, *rsum;
    int n_split, chunk_j, chunk_i;
};

static MfmaWs carve_mfma(void *ws, int64_t I, int64_t J, int64_t K) {
    MfmaWs w;
    w.n_split = kMfmaSplit;
    w.chunk_j = (int)(((J + kMfmaSplit - 1) / kMfmaSplit + 31) / 32 * 32);
    w.chunk_i = (int)(((I + kMfmaSplit - 1) / kMfmaSplit + 31) / 32 * 32);
    char *p = static_cast<char *>(ws);
    auto take = [&](size_t bytes) { float *r = reinterpret_cast<float *>(p); p += align256(bytes); return r; };
    w.rowv = take((size_t)I * 16);
    w.nb = take((size_t)J * 4);
    w.Ppart = take((size_t)kMfmaSplit * I * K * 4);
    w.Tpart = take((size_t)kMfmaSplit * J * K * 4);
    w.rowp = take((size_t)kMfmaSplit * 2 * I * 4);
    w.colp = take((size_t)kMfmaSplit * J * 4);
    w.rsum = take((size_t)I * 4);
    return w;
}

static int prep(const tad_plan &pl, const void *const *args, const MfmaWs &w, hipStream_t s) {
    const int I = (int)pl.fast.I, J = (int)pl.fast.J, K = (int)pl.fast.K;
    TAD_LAUNCH("k_mfma_prep", k_mfma_prep, dim3((I + J + 3) / 4), dim3(256), 0, s, (const float *)args[0],
               (const float *)args[1], (const float *)args[2], (const float *)args[3], w.rowv, w.nb, I, J, K,
               (int)pl.fast.c_ld);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

// ---------------------------------------------------------------------------------------------
// The same forward pass in the direct form  s_ij = sum_k (a_ik + b_jk)^2  on the vector ALUs (one add and one fused
// multiply-add per (i, j, k): 2 I J K lane operations): block tile 64 x 64, a
// thread owns 4 x 4 results, k tile 32 through LDS.  Kept to measure the expanded form against (TAD_PLAN_DIRECT_FORM).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_worked_forward_direct(const float *__restrict__ a, const float *__restrict__ b,
                                                               const float *__restrict__ rowv, float *__restrict__ f,
                                                               int I, int J, int K) {
    __shared__ __attribute__((aligned(16))) float As[32][68];   // [k][row]
    __shared__ __attribute__((aligned(16))) float Bs[32][68];   // [k][row]: a thread reads four consecutive rows as one 16-byte load
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = 0.f;
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
        // 64 rows x 32 k of a and of b: 512 16-byte loads each, two per thread (K % 32 == 0)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int idx = tid + 256 * p, row = idx >> 3, kq = idx & 7;
            const float4v va = (i0 + row < I) ? *reinterpret_cast<const float4v *>(a + (size_t)(i0 + row) * K + k0 + 4 * kq) : zero4;
            const float4v vb = (j0 + row < J) ? *reinterpret_cast<const float4v *>(b + (size_t)(j0 + row) * K + k0 + 4 * kq) : zero4;
#pragma unroll
            for (int q = 0; q < 4; ++q) { As[4 * kq + q][row] = va[q]; Bs[4 * kq + q][row] = vb[q]; }
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            const float4v av = *reinterpret_cast<const float4v *>(&As[k][4 * ty]);
            const float4v bv = *reinterpret_cast<const float4v *>(&Bs[k][4 * tx]);
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    const float t = av[x] + bv[y];
                    acc[x][y] = fmaf(t, t, acc[x][y]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int i = i0 + 4 * ty + x, j = j0 + 4 * tx;
        if (i < I && j < J) {   // J % 4 == 0
            const float c = rowv[i * 4 + 1], D = rowv[i * 4 + 2];   // -log2e c_ii, -log2e D_i
            float4v o;
#pragma unroll
            for (int y = 0; y < 4; ++y) o[y] = __builtin_amdgcn_exp2f(fmaf(c, acc[x][y], D));
            *reinterpret_cast<float4v *>(f + (size_t)i * J + j) = o;
        }
    }
}

int mfma_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s) {
    const int I = (int)pl.fast.I, J = (int)pl.fast.J, K = (int)pl.fast.K;
    MfmaWs w = carve_mfma(ws, I, J, K);
    int rc = prep(pl, args, w, s);
    if (rc) return rc;
    if (pl.flags & TAD_PLAN_DIRECT_FORM) {
        TAD_LAUNCH("k_worked_forward_direct", k_worked_forward_direct, dim3((J + 63) / 64, (I + 63) / 64), dim3(256), 0, s,
                   (const float *)args[0], (const float *)args[1], w.rowv, (float *)f, I, J, K);
        return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
    }
    TAD_LAUNCH("k_mfma_forward", k_mfma_forward, dim3((J + 127) / 128, (I + 127) / 128), dim3(256), 0, s,
               (const float *)args[0], (const float *)args[1], w.rowv, w.nb, (float *)f, I, J, K);
    return hipGetLastError() == hipSuccess ? TAD_OK : TAD_EDEVICE;
}

int mfma_backward(const tad_plan &pl, const void *const *args, const void *f_, const void *df_, void *const *dx,
                  void *ws, hipStream_t s) {
    const int I = (int)pl.fast.I, J = (int)pl.fast.J, K = (int)pl.fast.K, c_ld = (int)pl.fast.c_ld;
    MfmaWs w = carve_mfma(ws, I, J, K);
    const float *a = (const float *)args[0], *b = (const float *)args[1], *d = (const float *)args[3];
    const float *f = (const float *)f_, *df = (const float *)df_;
    int rc = prep(pl, args, w, s);
    if (rc) return rc;
    const int nz = (K + 255) / 256;
    // the row pass always runs: r_i feeds da, dc and dd; the column pass only for db
    TAD_LAUNCH("k_mfma_backward", (k_mfma_backward<false>), dim3((I + 63) / 64, w.n_split, nz), dim3(256), 0, s, f, df,
               b, w.rowv, w.nb, w.Ppart, w.rowp, I, J, K, w.chunk_j);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dx[1]) {
        TAD_LAUNCH("k_mfma_backward", (k_mfma_backward<true>), dim3((J + 63) / 64, w.n_split, nz), dim3(256), 0, s, f,
                   df, a, w.rowv, w.nb, w.Tpart, w.colp, I, J, K, w.chunk_i);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    if (dx[2]) {
        const long long n = pl.arg_count[2];
        const int g = (int)std::min<long long>(16384, (n / 4 + 255) / 256 + 1);
        TAD_LAUNCH("k_fill_zero", k_mfma_fill_zero, dim3(g), dim3(256), 0, s, (float *)dx[2], n);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    const int br = (I + 3) / 4, bc = dx[1] ? (J + 3) / 4 : 0;
    TAD_LAUNCH("k_mfma_finish", k_mfma_finish, dim3(br + bc), dim3(256), 0, s, a, b, w.rowv, w.Ppart, w.Tpart,
               w.n_split, w.rowp, w.colp, (float *)dx[0], (float *)dx[1], (float *)dx[2], w.rsum, I, J, K, c_ld, br);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (dx[3]) {
        const int n_d = (int)pl.arg_count[3];
        TAD_LAUNCH("k_mfma_dd", k_mfma_dd, dim3((n_d + 3) / 4), dim3(256), 0, s, pl.fast.feas, pl.fast.flat[0],
                   pl.fast.dd_iy, pl.fast.dd_iz, d, w.rsum, (float *)dx[3], n_d);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

}  // namespace tad
