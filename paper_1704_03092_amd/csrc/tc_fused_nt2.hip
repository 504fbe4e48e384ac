// Instantiations of the fused kernel for operands with up to 2 term(s) (one-level Strassen).
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(2)
}  // namespace fused
}  // namespace tc
