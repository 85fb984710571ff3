// Backward-kernel instantiations: element type f16, head dim 96.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_f16_d96(const BwdLaunchArgs &a) { return launch_bwd<_Float16, 96>(a); }
}  // namespace tsdpa
