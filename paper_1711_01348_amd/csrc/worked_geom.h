// Tile geometry and workspace layout of the worked-expression kernels (host and device).
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

constexpr int kStridedDwElems = 1024;  // function elements per dw block of the strided family (multiple of 256)

constexpr int AD_BTI_ROWS = 64;   // rows per backward tile of the antidiagonal pattern
inline size_t antidiag_workspace_bytes(int64_t I, int64_t n_x) {
    return align256((size_t)((I + AD_BTI_ROWS - 1) / AD_BTI_ROWS) * (size_t)n_x * 4);
}

}  // namespace tad
