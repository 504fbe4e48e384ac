// Instantiations of the fused kernel for operands with up to 4 term(s) (two-level Strassen).
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(4)
}  // namespace fused
}  // namespace tc
