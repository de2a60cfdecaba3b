// Kernel instantiations for a diagonal A or B (Section 5.2).
#include "kernel_table.hpp"
namespace fg {
#define FG_DIAG_TILE(BM, BN, WGM, WGN, TAG)                                                        \
    FG_ENTRY_X(BM, BN, 64, 2, WGM, WGN, true, true, 1, 0, "gemm_diagA_n_" TAG),                \
    FG_ENTRY_X(BM, BN, 64, 2, WGM, WGN, true, false, 1, 0, "gemm_diagA_t_" TAG),               \
    FG_ENTRY_X(BM, BN, 64, 2, WGM, WGN, true, true, 2, 0, "gemm_t_diagB_" TAG),                \
    FG_ENTRY_X(BM, BN, 64, 2, WGM, WGN, false, true, 2, 0, "gemm_n_diagB_" TAG)
const KernelEntry *kernel_table_diag() {
    static const KernelEntry t[DIAG_TILE_COUNT * 4] = {
        FG_DIAG_TILE(256, 256, 2, 4, "256x256x64"),
        FG_DIAG_TILE(256, 128, 4, 2, "256x128x64"),
        FG_DIAG_TILE(128, 128, 2, 2, "128x128x64"),
        FG_DIAG_TILE(64, 64, 2, 2, "64x64x64"),
    };
    return t;
}
}  // namespace fg
