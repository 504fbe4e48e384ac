// Fused kernel family: up to 4 terms of A and of B, counted at run time.
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(4, 4, false)
}  // namespace fused
}  // namespace tc
