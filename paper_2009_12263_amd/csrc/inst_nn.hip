// Kernel instantiations for the layout pair "nn" (A K-contiguous: false, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE(kernel_table_nn, false, true, "nn")
}
