// Forward-kernel instantiations: element type bf16, head dim 160, K/V tiles of 32 rows.
#include "sdpa_fwd_inst.h"

namespace tsdpa {
int launch_bf16_d160_tn64(int tile_m, const LaunchArgs &a);
int launch_bf16_d160(int tile_m, int tile_n, const LaunchArgs &a)
{
    return launch_dispatch<__bf16, 160>(tile_m, tile_n, a, &launch_bf16_d160_tn64);
}
}  // namespace tsdpa
