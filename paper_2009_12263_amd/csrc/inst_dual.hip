// Kernel instantiations for planar-split dual-number products (Section 5.4: eps^2 = 0, three real products).
#include "kernel_table.hpp"
namespace fg {
#define FG_DUAL_TILE(BM, BN, WGM, WGN, TAG)                                                        \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, false, true, 0, 2, "dgemm_nn_" TAG),                    \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, false, false, 0, 2, "dgemm_nt_" TAG),                   \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, true, true, 0, 2, "dgemm_tn_" TAG),                     \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, true, false, 0, 2, "dgemm_tt_" TAG)
const KernelEntry *kernel_table_dual() {
    static const KernelEntry t[CTILE_COUNT * 4] = {
        FG_DUAL_TILE(256, 128, 4, 2, "256x128x32"),
        FG_DUAL_TILE(128, 128, 2, 2, "128x128x32"),
        FG_DUAL_TILE(64, 64, 2, 2, "64x64x32"),
    };
    return t;
}
}  // namespace fg
