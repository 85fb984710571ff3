// Backward-kernel instantiations: element type f16, head dim 64.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_f16_d64(const BwdLaunchArgs &a) { return launch_bwd<_Float16, 64>(a); }
}  // namespace tsdpa
