// Launch geometry and workspace layout shared by the host planner and the kernels: tile sizes of the specialised
// families, sizes of their per-tile partial sums, and how the plan-driven fallback kernels share long sums.
#pragma once
#include <cstddef>
#include <cstdint>

namespace tad {

constexpr int FWD_TI = 4;       // rows per forward block (1024 columns): 40.6 us at 8192^2 against 43 / 46 us with 8 / 2 rows
constexpr int BWD_TI = 256;     // rows per backward block
constexpr int BWD_TJ = 512;     // columns per backward block
constexpr int kWorkedMaxK = 8;  // longest summed index the direct (VALU) kernels are instantiated for

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// row partials [n_jt][K+2][I], column partials [n_it][K+1][J]
inline size_t worked_workspace_bytes(int64_t I, int64_t J, int64_t K) {
    size_t n_jt = (size_t)((J + BWD_TJ - 1) / BWD_TJ), n_it = (size_t)((I + BWD_TI - 1) / BWD_TI);
    return align256(n_jt * I * (K + 2) * 4) + align256(n_it * (K + 1) * J * 4);
}

// long summed index (MFMA family): number of chunks the collapsed contraction index is split in (4 leaves the
// chip under-filled: 133 / 117 us per contraction instead of 98 / 94)
constexpr int kMfmaSplit = 8;
inline size_t mfma_workspace_bytes(int64_t I, int64_t J, int64_t K) {
    return align256((size_t)I * 16) + align256((size_t)J * 4) + align256((size_t)kMfmaSplit * I * K * 4) +
           align256((size_t)kMfmaSplit * J * K * 4) + align256((size_t)kMfmaSplit * 2 * I * 4) +
           align256((size_t)kMfmaSplit * J * 4) + align256((size_t)I * 4);
}

// Fallback (generic and program) kernels.  The cooperative form (one block per gradient element) pays off when
// an element sums many terms: measured on the worked expression at 8192 x 8192 x 5, the gradients with 8192 and
// 40960 terms per element take 0.8 ms this way against 11 ms with one thread per element.
inline bool use_cooperative_gather(long long n_elements, double terms_total) {
    return n_elements <= (1ll << 22) && terms_total / (double)(n_elements > 0 ? n_elements : 1) >= 1024.0;
}
// One block per element leaves most of the chip idle when the gradient has few elements (a filter, a bias, a
// scalar): the terms of an element are then shared by `splits` blocks, whose fp64 partial sums go to the
// workspace and are added in ascending order by a finishing kernel.  About 1024 blocks in all, at least 2048
// terms per block, at most 256 blocks per element.
inline int cooperative_splits(long long n_elements, double terms_total) {
    if (n_elements <= 0 || n_elements >= 1024 || !use_cooperative_gather(n_elements, terms_total)) return 1;
    const long long want = (1024 + n_elements - 1) / n_elements;
    const long long most = (long long)(terms_total / (double)n_elements / 2048.0);
    long long sp = want < most ? want : most;
    if (sp > 256) sp = 256;
    return sp < 1 ? 1 : (int)sp;
}
// partial sums [n_elements][splits] (fp64), then one flag per element (0: a mask zeroes it)
inline size_t split_workspace_bytes(long long n_elements, int splits) {
    return splits > 1 ? align256((size_t)n_elements * (size_t)splits * 8) + align256((size_t)n_elements * 4) : 0;
}

constexpr int kStridedDwElems = 1024;  // function elements per dw block of the strided family, direct form (multiple of 256)

// Strided family: the tiled kernels stage contiguous slices of x (forward, dw) and of df (1 - f^2) (dx) in LDS.
//   ti  rows i of f per forward / dw block (0: the slice of x does not fit, direct kernels)
//   tp  rows p of x per dx wavefront       (0: the slice of f does not fit, direct kernel)
struct StridedTiling {
    int ti, tp;
    int x_slice;    // floats of LDS for the slice of x (with room for the alignment shift)
    int t_slice;    // floats of LDS for the slice of df (1 - f^2), per wavefront
};
constexpr int kStridedLdsFloats = 10240;   // 40 KiB per block: four blocks per compute unit
constexpr int kStridedMaxPerThread = 4;    // function elements per thread of a dw block
constexpr int kStridedWaveFloats = 1280;   // LDS of one wavefront of a dx block: its slice of df (1 - f^2)
inline StridedTiling strided_tiling(int64_t N, int64_t I, int64_t J, int64_t U, int64_t s, int64_t P, int64_t Q) {
    StridedTiling t{0, 0, 0, 0};
    // forward / dw: rows s*i0 .. s*(i0+ti-1)+U-1 of x, whole rows; prefer at least 1024 blocks
    for (int ti = 8; ti >= 1; --ti) {
        const int64_t slice = (s * (ti - 1) + U) * Q + 8;   // + alignment shift and the ragged last vector
        if (ti * J > 256 * kStridedMaxPerThread || slice > kStridedLdsFloats) continue;
        if (t.ti == 0) { t.ti = ti; t.x_slice = (int)slice; }
        if (N * ((I + ti - 1) / ti) >= 1024) { t.ti = ti; t.x_slice = (int)slice; break; }
    }
    // dx: a wavefront takes tp rows p and 64 columns q; the rows ceil((p0-U+1)/s) .. floor((p0+tp-1)/s) of f carry its
    // terms.  Whole rows of f between the first and the last term: (rows - 1) J + about 64 / s + U columns.
    for (int tp = 16; tp >= 1; --tp) {
        const int64_t rows = (tp - 1 + U - 1) / s + 2;
        const int64_t piece = (rows - 1) * J + 64 / s + U + 2 + 8;
        if (piece > kStridedWaveFloats) continue;
        t.tp = tp;
        t.t_slice = (int)kStridedWaveFloats;
        break;
    }
    (void)P;
    return t;
}
inline size_t strided_workspace_bytes(int64_t N, int64_t I, int64_t J, int64_t U, int64_t V, int64_t s, int64_t P, int64_t Q) {
    const StridedTiling t = strided_tiling(N, I, J, U, s, P, Q);
    const int64_t direct = (N * I * J + kStridedDwElems - 1) / kStridedDwElems;
    const int64_t tiled = t.ti ? N * ((I + t.ti - 1) / t.ti) : 0;
    return align256((size_t)(direct > tiled ? direct : tiled) * (size_t)(U * V) * 4);
}

// antidiagonal pattern, backward: aligned tiles of df; a tile yields AD_TILE_ROWS + AD_TILE_COLS antidiagonal sums
constexpr int AD_TILE_ROWS = 256, AD_TILE_COLS = 256, AD_TILE_SUMS = AD_TILE_ROWS + AD_TILE_COLS;
inline size_t antidiag_workspace_bytes(int64_t I, int64_t J) {
    return align256((size_t)((I + AD_TILE_ROWS - 1) / AD_TILE_ROWS) * (size_t)((J + AD_TILE_COLS - 1) / AD_TILE_COLS) *
                    AD_TILE_SUMS * 4);
}

}  // namespace tad
