// bfloat16 kernel instantiations for the layout pair "nt" (A K-contiguous: false, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_BF16(kernel_table_nt_bf16, false, false, "nt")
}
