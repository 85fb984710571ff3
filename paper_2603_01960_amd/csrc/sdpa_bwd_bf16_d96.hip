// Backward-kernel instantiations: element type bf16, head dim 96.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_bf16_d96(const BwdLaunchArgs &a) { return launch_bwd<__bf16, 96>(a); }
}  // namespace tsdpa
