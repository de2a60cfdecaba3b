// Kernel instantiations with element-wise addition on loaded A and B values, layout pair "nt"
// (A K-contiguous: false, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_XF(kernel_table_nt_xf, false, false, "nt")
}
