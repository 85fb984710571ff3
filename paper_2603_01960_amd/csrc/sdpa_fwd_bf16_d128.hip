// Forward-kernel instantiations: element type bf16, head dim 128, K/V tiles of 32 rows.
#include "sdpa_fwd_inst.h"

namespace tsdpa {
int launch_bf16_d128_tn64(int tile_m, const LaunchArgs &a);
int launch_bf16_d128(int tile_m, int tile_n, const LaunchArgs &a)
{
    return launch_dispatch<__bf16, 128>(tile_m, tile_n, a, &launch_bf16_d128_tn64);
}
}  // namespace tsdpa
