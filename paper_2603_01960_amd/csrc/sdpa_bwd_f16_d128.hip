// Backward-kernel instantiations: element type f16, head dim 128.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_f16_d128(const BwdLaunchArgs &a) { return launch_bwd<_Float16, 128>(a); }
}  // namespace tsdpa
