// Backward-kernel instantiations: element type bf16, head dim 160.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_bf16_d160(const BwdLaunchArgs &a) { return launch_bwd<__bf16, 160>(a); }
}  // namespace tsdpa
