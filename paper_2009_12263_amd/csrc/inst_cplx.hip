// Kernel instantiations for planar-split complex products (Section 5.4).
#include "kernel_table.hpp"
namespace fg {
#define FG_CPLX_TILE(BM, BN, WGM, WGN, TAG)                                                        \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, false, true, 0, 1, "cgemm_nn_" TAG),                    \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, false, false, 0, 1, "cgemm_nt_" TAG),                   \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, true, true, 0, 1, "cgemm_tn_" TAG),                     \
    FG_ENTRY_X(BM, BN, 32, 2, WGM, WGN, true, false, 0, 1, "cgemm_tt_" TAG)
const KernelEntry *kernel_table_cplx() {
    static const KernelEntry t[CTILE_COUNT * 4] = {
        FG_CPLX_TILE(256, 128, 4, 2, "256x128x32"),
        FG_CPLX_TILE(128, 128, 2, 2, "128x128x32"),
        FG_CPLX_TILE(64, 64, 2, 2, "64x64x32"),
    };
    return t;
}
}  // namespace fg
