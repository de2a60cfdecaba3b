// Kernel instantiations with element-wise addition on loaded A and B values, layout pair "nn"
// (A K-contiguous: false, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_XF(kernel_table_nn_xf, false, true, "nn")
}
