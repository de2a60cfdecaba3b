// Kernel instantiations for the layout pair "tt" (A K-contiguous: true, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE(kernel_table_tt, true, false, "tt")
}
