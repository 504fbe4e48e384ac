// Instantiations of the fused kernel for operands with up to 1 term(s) (classical mode, dense temporaries).
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(1)
}  // namespace fused
}  // namespace tc
