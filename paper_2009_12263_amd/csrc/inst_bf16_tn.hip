// bfloat16 kernel instantiations for the layout pair "tn" (A K-contiguous: true, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_BF16(kernel_table_tn_bf16, true, true, "tn")
}
