// Forward-kernel instantiations: element type f16, head dim 96, K/V tiles of 64 rows.
#include "sdpa_fwd_inst.h"

namespace tsdpa {
int launch_f16_d96_tn64(int tile_m, const LaunchArgs &a) { return launch_dispatch_tn64<_Float16, 96>(tile_m, a); }
}  // namespace tsdpa
