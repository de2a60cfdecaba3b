// Kernel instantiations with element-wise addition on loaded A and B values, layout pair "tt"
// (A K-contiguous: true, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_XF(kernel_table_tt_xf, true, false, "tt")
}
