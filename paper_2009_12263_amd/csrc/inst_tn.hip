// Kernel instantiations for the layout pair "tn" (A K-contiguous: true, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE(kernel_table_tn, true, true, "tn")
}
