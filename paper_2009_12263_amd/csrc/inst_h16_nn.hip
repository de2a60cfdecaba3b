// Kernel instantiations with binary16 C and D for the layout pair "nn" (A K-contiguous: false, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_H16(kernel_table_nn_h16, false, true, "nn")
}
