// Fused kernel, small geometry, products whose operand sums have one block each.
#include "tc_fused_small.h"
namespace tc {
namespace fused_small {
TC_FUSED_DEFINE_LAUNCH(1, 1, true)
}
}  // namespace tc
