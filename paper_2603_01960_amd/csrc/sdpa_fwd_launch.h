// Host-side launch plumbing shared by the per-(dtype, D) instantiation files and the C-ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsdpa {

struct LaunchArgs {
    const void *q, *k, *v;
    void *o;
    float *lse;
    int BH, S;
    float c;          // |scale| * log2(e)
    float tau;        // lazy-rescale threshold in log2 units (0 = raise the reference on every new maximum)
    uint32_t qsign;   // 0x80008000 when scale < 0 (sign folded into Q), else 0
    int linear_grid;
    int causal;       // causal mask (Section 4.1.3): key j contributes to query i only if j <= i + Skv - S
    int kv;           // 0: S queries against the same S keys.  1: the general kernel (Skv keys, split key range)
    int Skv;          // key/value rows per head (kv = 1)
    int splits;       // workgroups per (head, query tile) along the key axis (kv = 1); > 1 writes partials to ws
    float *ws;        // split workspace: float [BH][splits][S][D] then [BH][splits][S][2]
    hipStream_t stream;
};

// Each returns a hipError_t cast to int (0 = success); tile_m in {64,128}, tile_n in {32,64,128}
// (tile_n in {32,64} when a.kv is set).
int launch_f16_d64(int tile_m, int tile_n, const LaunchArgs &a);
int launch_f16_d96(int tile_m, int tile_n, const LaunchArgs &a);
int launch_f16_d128(int tile_m, int tile_n, const LaunchArgs &a);
int launch_f16_d160(int tile_m, int tile_n, const LaunchArgs &a);
int launch_bf16_d64(int tile_m, int tile_n, const LaunchArgs &a);
int launch_bf16_d96(int tile_m, int tile_n, const LaunchArgs &a);
int launch_bf16_d128(int tile_m, int tile_n, const LaunchArgs &a);
int launch_bf16_d160(int tile_m, int tile_n, const LaunchArgs &a);

}  // namespace tsdpa
