// Contraction of two matrices over one summation index (Sec. 5, example f^4_ij = sum_k x_ik y_kj, and Sec. 5.2):
// body "mul" with two function indices and one summation index, fp32.  In the gather form every gradient
// element owns one kernel coordinate that runs over a whole dimension with constant limits (the collapsed
// function index), so forward pass and both gradients are dense matrix products,
//
//     f  = P Q          dP = df Q^T          dQ = P^T df
//
// (P: the operand indexed by the first function index and the summation index, Q: the other one; either may be
// stored with its two axes in either order).  They run on the matrix cores (v_mfma_f32_32x32x2f32).
//
// One kernel, C[m][n] = sum_k A(m, k) B(k, n), with the memory order of each operand a template parameter:
//   AT = false: A(m, k) = a[m * lda + k]      AT = true: A(m, k) = a[k * lda + m]
//   BT = false: B(k, n) = b[k * ldb + n]      BT = true: B(k, n) = b[n * ldb + k]
// Block tile 128 x 128, four waves of 64 x 64 (2 x 2 MFMA tiles), contraction tile 32, global -> register -> LDS
// staging.  Two sets of tiles in LDS: while the MFMAs of tile t read one set, the registers holding tile t + 1 are
// written to the other set and the global loads of tile t + 2 go out, all of it between MFMA groups, so that one
// barrier per tile remains and no wave stands idle while a tile is staged.  Every vector-ALU instruction issued on
// a SIMD takes about four cycles from its matrix core (measured: 4 / 8 / 16 extra v_add per group of four MFMAs
// lengthen the group by 14 / 26 / 61 cycles; LDS and scalar instructions cost nothing), so a workgroup whose tiles lie
// wholly inside the operands runs a loop with next to no vector-ALU work: two tiles per pass, so that the LDS set is
// a constant and every LDS address is one per-lane base plus an immediate; global addresses are a uniform base,
// advanced on the scalar unit, plus a constant 32-bit offset per thread; no bounds checks, no zero fill (about 20
// instead of 85 vector-ALU instructions per 64 MFMAs).  Workgroups on a ragged edge take the checked loop.  A product with few
// output tiles and a long contraction index is cut along that index (blockIdx.y): every piece writes its partial
// product to the workspace and k_contract_reduce adds the pieces in a fixed order.
//
// MFMA operand layout (wave64): A operand lane l = A[m = l % 32][k = l / 32], B operand lane l = B[k = l / 32][n = l % 32],
// result register r of lane l = D[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].
#include <hip/hip_runtime.h>

#include <type_traits>

#include "launch.h"
#include "profile.h"

namespace tad {

typedef float float4c __attribute__((ext_vector_type(4)));
typedef float float16c __attribute__((ext_vector_type(16)));

constexpr int CT_KT = 32;        // contraction tile
constexpr int CT_LDK = 33;       // row stride of a [row][k] tile: odd, conflict-free 4-byte reads down a column of rows
constexpr int CT_LDM = 132;      // row stride of a [k][row] tile: 16-byte aligned rows
constexpr int CT_TILE = 128 * CT_LDK;   // floats per operand tile; 32 * CT_LDM is the same size
static_assert(32 * CT_LDM == CT_TILE, "both tile layouts use the same amount of LDS");

// The 8 accelerator dies take workgroups round robin; give each die a contiguous range of logical tiles and walk
// the tiles in groups of 8 tile rows so that concurrently running workgroups share operand tiles in their L2.
__device__ __forceinline__ void tile_of_block(int gm, int gn, int &tm, int &tn) {
    const int total = gm * gn;
    int lid = blockIdx.x;
    if (total % 8 == 0) lid = (lid % 8) * (total / 8) + lid / 8;
    const int group = 8 * gn;
    const int g0 = (lid / group) * 8;
    const int rows = min(8, gm - g0);
    const int in = lid - (lid / group) * group;
    tm = g0 + in % rows;
    tn = in / rows;
}

template <bool AT, bool BT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k_contract(const float *__restrict__ a, const float *__restrict__ b, float *__restrict__ c, int M, int N, int Kc,
                int lda, int ldb, int gm, int gn, int chunk, int lean_ok) {
    __shared__ __attribute__((aligned(16))) float smem[4 * CT_TILE];   // two sets of (A tile, B tile); reused as the output stage in the epilogue
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of_block(gm, gn, tm, tn);
    const int m0 = tm * 128, n0 = tn * 128;
    // this workgroup's piece of the contraction index (chunk is a multiple of the tile; one piece: chunk >= Kc)
    const int kb = blockIdx.y * chunk;
    Kc = min(Kc, kb + chunk);
    c += (size_t)blockIdx.y * M * N;
    float16c acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;
    float4c ra[4], rb[4];
    const int mrow = lane & 31, kof = lane >> 5;
    // lean_ok (host): the 32-bit byte offsets below cannot overflow
    if (lean_ok && m0 + 128 <= M && n0 + 128 <= N && (Kc - kb) % CT_KT == 0) {   // the same for the whole workgroup
        // global: thread -> (row, 4 consecutive k) or (k, 4 consecutive rows); part p adds 32 rows / 8 values of k
        const unsigned ga = !AT ? (unsigned)(((tid >> 3) * lda + 4 * (tid & 7)) * 4) : (unsigned)(((tid >> 5) * lda + 4 * (tid & 31)) * 4);
        const unsigned gb = BT ? (unsigned)(((tid >> 3) * ldb + 4 * (tid & 7)) * 4) : (unsigned)(((tid >> 5) * ldb + 4 * (tid & 31)) * 4);
        const unsigned gpa = (!AT ? 32u : 8u) * (unsigned)lda * 4u, gpb = (BT ? 32u : 8u) * (unsigned)ldb * 4u;
        const char *pa = reinterpret_cast<const char *>(!AT ? a + (size_t)m0 * lda + kb : a + (size_t)kb * lda + m0);
        const char *pb = reinterpret_cast<const char *>(BT ? b + (size_t)n0 * ldb + kb : b + (size_t)kb * ldb + n0);
        const size_t stepa = (!AT ? (size_t)CT_KT : (size_t)CT_KT * lda) * 4, stepb = (BT ? (size_t)CT_KT : (size_t)CT_KT * ldb) * 4;
        auto gload = [&]() {   // the tile at pa, pb; then on to the next one
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                ra[p] = *reinterpret_cast<const float4c *>(pa + (ga + p * gpa));
                rb[p] = *reinterpret_cast<const float4c *>(pb + (gb + p * gpb));
            }
            pa += stepa;
            pb += stepb;
        };
        // LDS: one base per lane for the writes of each operand and one for its reads
        const int wa = !AT ? (tid >> 3) * CT_LDK + 4 * (tid & 7) : (tid >> 5) * CT_LDM + 4 * (tid & 31);
        const int wb = CT_TILE + (BT ? (tid >> 3) * CT_LDK + 4 * (tid & 7) : (tid >> 5) * CT_LDM + 4 * (tid & 31));
        const int rda = !AT ? (wm * 64 + mrow) * CT_LDK + kof : kof * CT_LDM + wm * 64 + mrow;
        const int rdb = CT_TILE + (BT ? (wn * 64 + mrow) * CT_LDK + kof : kof * CT_LDM + wn * 64 + mrow);
        auto stage = [&](auto SET) {
            constexpr int so = decltype(SET)::value * 2 * CT_TILE;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (!AT) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) smem[wa + so + p * 32 * CT_LDK + q] = ra[p][q];
                } else {
                    *reinterpret_cast<float4c *>(&smem[wa + so + p * 8 * CT_LDM]) = ra[p];
                }
                if (BT) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) smem[wb + so + p * 32 * CT_LDK + q] = rb[p][q];
                } else {
                    *reinterpret_cast<float4c *>(&smem[wb + so + p * 8 * CT_LDM]) = rb[p];
                }
            }
        };
        auto tile = [&](auto SET, bool more1, bool more2) {
            constexpr int set = decltype(SET)::value, so = set * 2 * CT_TILE;
            auto afrag = [&](int kk, int half) -> float { return smem[rda + so + (!AT ? 32 * half * CT_LDK + kk : kk * CT_LDM + 32 * half)]; };
            auto bfrag = [&](int kk, int half) -> float { return smem[rdb + so + (BT ? 32 * half * CT_LDK + kk : kk * CT_LDM + 32 * half)]; };
            float a0 = afrag(0, 0), a1 = afrag(0, 1), b0 = bfrag(0, 0), b1 = bfrag(0, 1);
#pragma unroll
            for (int ks = 0; ks < CT_KT / 2; ++ks) {
                float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
                if (ks + 1 < CT_KT / 2) {
                    na0 = afrag(2 * ks + 2, 0);
                    na1 = afrag(2 * ks + 2, 1);
                    nb0 = bfrag(2 * ks + 2, 0);
                    nb1 = bfrag(2 * ks + 2, 1);
                }
                if (ks == 1 && more1) stage(std::integral_constant<int, set ^ 1>{});
                if (ks == 3 && more2) gload();
                __builtin_amdgcn_sched_barrier(0);
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
            }
            __syncthreads();
        };
        const int nt = (Kc - kb) / CT_KT;   // >= 1: no piece is empty
        gload();
        stage(std::integral_constant<int, 0>{});
        __syncthreads();
        if (nt > 1) gload();
        for (int t = 0; t < nt; t += 2) {
            tile(std::integral_constant<int, 0>{}, t + 1 < nt, t + 2 < nt);
            if (t + 1 < nt) tile(std::integral_constant<int, 1>{}, t + 2 < nt, t + 3 < nt);
        }
    } else {
        const float4c zero4 = {0.f, 0.f, 0.f, 0.f};
        // every dimension is a multiple of 4 (checked on the host): a 16-byte load is inside or outside as a whole
        auto gload = [&](int k0) {
    #pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int idx = tid + 256 * p;
                if (!AT) {
                    const int row = idx >> 3, kq = idx & 7;
                    const int m = m0 + row, k = k0 + 4 * kq;
                    ra[p] = (m < M && k < Kc) ? *reinterpret_cast<const float4c *>(a + (size_t)m * lda + k) : zero4;
                } else {
                    const int kk = idx >> 5, mq = idx & 31;
                    const int m = m0 + 4 * mq, k = k0 + kk;
                    ra[p] = (m < M && k < Kc) ? *reinterpret_cast<const float4c *>(a + (size_t)k * lda + m) : zero4;
                }
                if (BT) {
                    const int row = idx >> 3, kq = idx & 7;
                    const int n = n0 + row, k = k0 + 4 * kq;
                    rb[p] = (n < N && k < Kc) ? *reinterpret_cast<const float4c *>(b + (size_t)n * ldb + k) : zero4;
                } else {
                    const int kk = idx >> 5, nq = idx & 31;
                    const int n = n0 + 4 * nq, k = k0 + kk;
                    rb[p] = (n < N && k < Kc) ? *reinterpret_cast<const float4c *>(b + (size_t)k * ldb + n) : zero4;
                }
            }
        };
        auto stage = [&](int set) {
            float *As = smem + set * (2 * CT_TILE), *Bs = As + CT_TILE;
    #pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int idx = tid + 256 * p;
                if (!AT) {
                    const int row = idx >> 3, kq = idx & 7;
    #pragma unroll
                    for (int q = 0; q < 4; ++q) As[row * CT_LDK + 4 * kq + q] = ra[p][q];
                } else {
                    const int kk = idx >> 5, mq = idx & 31;
                    *reinterpret_cast<float4c *>(&As[kk * CT_LDM + 4 * mq]) = ra[p];
                }
                if (BT) {
                    const int row = idx >> 3, kq = idx & 7;
    #pragma unroll
                    for (int q = 0; q < 4; ++q) Bs[row * CT_LDK + 4 * kq + q] = rb[p][q];
                } else {
                    const int kk = idx >> 5, nq = idx & 31;
                    *reinterpret_cast<float4c *>(&Bs[kk * CT_LDM + 4 * nq]) = rb[p];
                }
            }
        };
        auto afrag = [&](int set, int kk, int half) -> float {
            const float *As = smem + set * (2 * CT_TILE);
            const int m = wm * 64 + 32 * half + mrow;
            return AT ? As[(kk + kof) * CT_LDM + m] : As[m * CT_LDK + kk + kof];
        };
        auto bfrag = [&](int set, int kk, int half) -> float {
            const float *Bs = smem + set * (2 * CT_TILE) + CT_TILE;
            const int n = wn * 64 + 32 * half + mrow;
            return BT ? Bs[n * CT_LDK + kk + kof] : Bs[(kk + kof) * CT_LDM + n];
        };
        gload(kb);
        stage(0);
        __syncthreads();
        if (kb + CT_KT < Kc) gload(kb + CT_KT);
        int set = 0;
        for (int k0 = kb; k0 < Kc; k0 += CT_KT, set ^= 1) {
            // the operands of step ks + 1 are read from LDS before the MFMAs of step ks are issued
            float a0 = afrag(set, 0, 0), a1 = afrag(set, 0, 1), b0 = bfrag(set, 0, 0), b1 = bfrag(set, 0, 1);
    #pragma unroll
            for (int ks = 0; ks < CT_KT / 2; ++ks) {
                float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
                if (ks + 1 < CT_KT / 2) {
                    na0 = afrag(set, 2 * ks + 2, 0);
                    na1 = afrag(set, 2 * ks + 2, 1);
                    nb0 = bfrag(set, 2 * ks + 2, 0);
                    nb1 = bfrag(set, 2 * ks + 2, 1);
                }
                // between MFMA groups: tile t + 1 goes from the registers to the other set (nobody reads that set any
                // more: the barrier at the end of tile t - 1), then the loads of tile t + 2 go out
                if (ks == 1 && k0 + CT_KT < Kc) stage(set ^ 1);
                if (ks == 3 && k0 + 2 * CT_KT < Kc) gload(k0 + 2 * CT_KT);
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
    }
    // epilogue: each wave stages 32 x 64 results at a time in its own quarter of the tile memory (32 rows of 66
    // floats) and writes them as 16-byte stores, 256 bytes per row.  The last barrier of the loop guarantees that
    // nobody still reads the tiles; a wave reads back only what it wrote itself.
    static_assert(4 * 32 * 66 <= 4 * CT_TILE, "output stage does not fit in the tile memory");
    float *out = smem + wave * (32 * 66);
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int mloc = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                out[mloc * 66 + y * 32 + mrow] = acc[x][y][r];
            }
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int rl = it * 4 + (lane >> 4), cl = (lane & 15) * 4;
            const int m = m0 + wm * 64 + x * 32 + rl, n = n0 + wn * 64 + cl;
            if (m < M && n < N) {
                const float4c v = {out[rl * 66 + cl], out[rl * 66 + cl + 1], out[rl * 66 + cl + 2], out[rl * 66 + cl + 3]};
                *reinterpret_cast<float4c *>(c + (size_t)m * N + n) = v;
            }
        }
    }
}

// c[i] = sum over the pieces of part[piece * n + i], pieces added in ascending order (n is a multiple of 4)
__global__ __launch_bounds__(256) void k_contract_reduce(const float *__restrict__ part, float *__restrict__ c,
                                                         long long n4, int pieces) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const float4c *src = reinterpret_cast<const float4c *>(part);
    float4c acc = src[i];
    for (int p = 1; p < pieces; ++p) acc += src[(long long)p * n4 + i];
    reinterpret_cast<float4c *>(c)[i] = acc;
}

static int launch_gemm(const GemmDesc &g, const float *a, const float *b, float *c, float *ws, hipStream_t s) {
    const int gm = (g.M + 127) / 128, gn = (g.N + 127) / 128;
    const int pieces = (g.splits > 1 && ws) ? g.splits : 1;
    // whole tiles per piece; the last piece may be shorter, none is empty
    const int chunk = pieces > 1 ? ((g.Kc + pieces - 1) / pieces + CT_KT - 1) / CT_KT * CT_KT : g.Kc;
    const int used = pieces > 1 ? (g.Kc + chunk - 1) / chunk : 1;
    const dim3 grid(gm * gn, used), block(256);
    // the lean loop addresses a tile's rows with 32-bit byte offsets
    const int lean_ok = (long long)g.lda * 128 * 4 < (1ll << 31) && (long long)g.ldb * 128 * 4 < (1ll << 31) ? 1 : 0;
    float *dst = used > 1 ? ws : c;
    if (!g.at && !g.bt)
        TAD_LAUNCH("k_contract", (k_contract<false, false>), grid, block, 0, s, a, b, dst, g.M, g.N, g.Kc, g.lda, g.ldb, gm, gn, chunk, lean_ok);
    else if (!g.at && g.bt)
        TAD_LAUNCH("k_contract", (k_contract<false, true>), grid, block, 0, s, a, b, dst, g.M, g.N, g.Kc, g.lda, g.ldb, gm, gn, chunk, lean_ok);
    else if (g.at && !g.bt)
        TAD_LAUNCH("k_contract", (k_contract<true, false>), grid, block, 0, s, a, b, dst, g.M, g.N, g.Kc, g.lda, g.ldb, gm, gn, chunk, lean_ok);
    else
        TAD_LAUNCH("k_contract", (k_contract<true, true>), grid, block, 0, s, a, b, dst, g.M, g.N, g.Kc, g.lda, g.ldb, gm, gn, chunk, lean_ok);
    if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    if (used > 1) {
        const long long n4 = (long long)g.M * g.N / 4;
        TAD_LAUNCH("k_contract_reduce", k_contract_reduce, dim3((unsigned)((n4 + 255) / 256)), block, 0, s, ws, c, n4, used);
        if (hipGetLastError() != hipSuccess) return TAD_EDEVICE;
    }
    return TAD_OK;
}

// source -1 of a product is df, destination -1 is f
int contract_forward(const tad_plan &pl, const void *const *args, void *f, void *ws, hipStream_t s) {
    const GemmDesc &g = pl.fast.gemm[0];
    return launch_gemm(g, (const float *)args[g.a_src], (const float *)args[g.b_src], (float *)f, (float *)ws, s);
}

int contract_backward(const tad_plan &pl, const void *const *args, const void *df, void *const *dx, void *ws,
                      hipStream_t s) {
    for (int q = 1; q <= 2; ++q) {
        const GemmDesc &g = pl.fast.gemm[q];
        if (!dx[g.out]) continue;
        const float *a = g.a_src < 0 ? (const float *)df : (const float *)args[g.a_src];
        const float *b = g.b_src < 0 ? (const float *)df : (const float *)args[g.b_src];
        const int rc = launch_gemm(g, a, b, (float *)dx[g.out], (float *)ws, s);   // the products share the workspace in turn
        if (rc) return rc;
    }
    return TAD_OK;
}

}  // namespace tad
