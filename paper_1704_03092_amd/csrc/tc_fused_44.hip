// Fused kernel family: 4 term(s) of A, 4 of B, exact.
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(4, 4, true)
}  // namespace fused
}  // namespace tc
