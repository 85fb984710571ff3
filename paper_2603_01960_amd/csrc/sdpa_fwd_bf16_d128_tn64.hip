// Forward-kernel instantiations: element type bf16, head dim 128, K/V tiles of 64 rows.
#include "sdpa_fwd_inst.h"

namespace tsdpa {
int launch_bf16_d128_tn64(int tile_m, const LaunchArgs &a) { return launch_dispatch_tn64<__bf16, 128>(tile_m, a); }
}  // namespace tsdpa
