"""MI355X-native tiled SDPA (online softmax, streamed K/V tiles): forward, split-KV / decoding shapes, backward.

The compute path is the HIP library ``libtiled_sdpa.so`` built from ``csrc/``;
:mod:`.binding` marshals torch tensors to its C-ABI.  :mod:`.workloads` only
draws seeded inputs.
"""
from .binding import (  # noqa: F401
    F16, BF16, TiledSdpaError, bwd_workspace_bytes, sdpa_backward, tiled_sdpa_bwd, kv_default_splits, kv_workspace_bytes, library_path, load_library,
    probe_mfma, probe_hbm_read, tune_tile, sdpa, sdpa_kv, sdpa_paged, status_string, tiled_sdpa_fwd, tiled_sdpa_fwd_ex, tiled_sdpa_fwd_kv,
    tiled_sdpa_fwd_gqa, tiled_sdpa_fwd_kvcache, tiled_sdpa_fwd_kvcache_static, tiled_sdpa_fwd_paged, version,
)
