// Fused kernel family: 4 term(s) of A, 4 of B at most, counted at run time.
#include "tc_fused.h"

namespace tc {
namespace fused {
TC_FUSED_DEFINE_LAUNCH(4, 4, false)
}  // namespace fused
}  // namespace tc
