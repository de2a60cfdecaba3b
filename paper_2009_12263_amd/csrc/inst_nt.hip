// Kernel instantiations for the layout pair "nt" (A K-contiguous: false, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE(kernel_table_nt, false, false, "nt")
}
