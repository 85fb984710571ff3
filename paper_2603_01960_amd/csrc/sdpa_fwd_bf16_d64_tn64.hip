// Forward-kernel instantiations: element type bf16, head dim 64, K/V tiles of 64 rows.
#include "sdpa_fwd_inst.h"

namespace tsdpa {
int launch_bf16_d64_tn64(int tile_m, const LaunchArgs &a) { return launch_dispatch_tn64<__bf16, 64>(tile_m, a); }
}  // namespace tsdpa
