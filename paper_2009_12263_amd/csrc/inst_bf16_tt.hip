// bfloat16 kernel instantiations for the layout pair "tt" (A K-contiguous: true, B K-contiguous: false).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_BF16(kernel_table_tt_bf16, true, false, "tt")
}
