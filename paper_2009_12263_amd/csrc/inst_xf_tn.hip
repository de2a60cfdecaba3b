// Kernel instantiations with element-wise addition on loaded A and B values, layout pair "tn"
// (A K-contiguous: true, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_XF(kernel_table_tn_xf, true, true, "tn")
}
