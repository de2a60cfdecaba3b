// bfloat16 kernel instantiations for the layout pair "nn" (A K-contiguous: false, B K-contiguous: true).
#include "kernel_table.hpp"
namespace fg {
FG_DEFINE_TABLE_BF16(kernel_table_nn_bf16, false, true, "nn")
}
