// Kernel instantiations for complex products on interleaved storage (Section 5.4: interleaved in
// global memory, split in shared memory; the conversion happens in the global-to-shared copy).
#include "kernel_table.hpp"
namespace fg {
#define FG_IL_TILE(BM, BN, WGM, WGN, TAG)                                                          \
    FG_ENTRY_IL(BM, BN, 32, 2, WGM, WGN, false, true, "cgemm_il_nn_" TAG),                         \
    FG_ENTRY_IL(BM, BN, 32, 2, WGM, WGN, false, false, "cgemm_il_nt_" TAG),                        \
    FG_ENTRY_IL(BM, BN, 32, 2, WGM, WGN, true, true, "cgemm_il_tn_" TAG),                          \
    FG_ENTRY_IL(BM, BN, 32, 2, WGM, WGN, true, false, "cgemm_il_tt_" TAG)
const KernelEntry *kernel_table_cplx_il() {
    static const KernelEntry t[CTILE_COUNT * 4] = {
        FG_IL_TILE(256, 128, 4, 2, "256x128x32"),
        FG_IL_TILE(128, 128, 2, 2, "128x128x32"),
        FG_IL_TILE(64, 64, 2, 2, "64x64x32"),
    };
    return t;
}
}  // namespace fg
