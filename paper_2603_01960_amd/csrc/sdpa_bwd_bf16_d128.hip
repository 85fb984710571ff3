// Backward-kernel instantiations: element type bf16, head dim 128.
#include "sdpa_bwd_inst.h"

namespace tsdpa {
int launch_bwd_bf16_d128(const BwdLaunchArgs &a) { return launch_bwd<__bf16, 128>(a); }
}  // namespace tsdpa
