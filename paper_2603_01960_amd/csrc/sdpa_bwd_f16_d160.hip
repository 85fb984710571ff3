// Backward-kernel instantiations: element type f16, head dim 160.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_f16_d160(const BwdLaunchArgs &a) { return launch_bwd<_Float16, 160>(a); }
}  // namespace tsdpa
