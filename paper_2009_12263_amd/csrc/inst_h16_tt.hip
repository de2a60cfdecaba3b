// Kernel instantiations with binary16 C and D for the layout pair "tt" (A K-contiguous: true, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_H16(kernel_table_tt_h16, true, false, "tt")
}
