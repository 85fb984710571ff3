// Backward-kernel instantiations: element type bf16, head dim 64.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_bf16_d64(const BwdLaunchArgs &a) { return launch_bwd<__bf16, 64>(a); }
}  // namespace tsdpa
