// Kernel instantiations with binary16 C and D for the layout pair "tn" (A K-contiguous: true, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_H16(kernel_table_tn_h16, true, true, "tn")
}
