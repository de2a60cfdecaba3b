// Kernel instantiations with binary16 C and D for the layout pair "nt" (A K-contiguous: false, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_H16(kernel_table_nt_h16, false, false, "nt")
}
