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
    const int *kv_lens;   // kv = 1: NULL, or valid key rows per batch entry (device, int32 [B]); Skv is then the capacity
    int heads_per_batch;  // kv = 1: key/value heads per batch entry (head / heads_per_batch indexes kv_lens)
    const int *block_table; // kv = 1: NULL, or pages of a paged cache (device, int32 [B][max_blocks]); k, v are then [pages][heads_per_batch][1 << block_shift][D]
    int max_blocks, block_shift;
    int tile_rot;      // kv = 1, dense cache: 1 = every workgroup starts its sweep over the unmasked tiles at a tile of its own
    int rows_per_head; // kv = 1: query positions per query head; S / rows_per_head query heads are folded into the S rows
    hipStream_t stream;
};

// Rows of slack after the B*H*S entries of each backward statistics array: the keys-resident pass
// reads them 4 rows at a time up to a tile past the last row of the last head.
constexpr int kBwdStatPad = 128;

struct BwdLaunchArgs {
    const void *q, *k, *v, *o, *dout;
    const float *lse;        // natural-log LSE of the forward pass, [BH, S]
    void *dq, *dk, *dv;
    float *delta, *lse2;     // workspace halves: [BH*S + slack] each
    unsigned stat_bytes;     // bytes of one workspace half
    int BH, S;               // query heads (B * H) and rows per head
    int group;               // query heads per key/value head (1: k, v, dk, dv have BH heads too; else BH / group)
    float c;                 // |scale| * log2(e)
    float scale;             // signed scale: factor of dQ and dK
    uint32_t rsign;          // 0x80008000 when scale < 0 (sign folded into the resident Q or K), else 0
    int causal;
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


// Backward pass: statistics kernel, then the dV, dK (keys resident) and dQ (queries resident) passes.
int launch_bwd_f16_d64(const BwdLaunchArgs &a);
int launch_bwd_f16_d96(const BwdLaunchArgs &a);
int launch_bwd_f16_d128(const BwdLaunchArgs &a);
int launch_bwd_f16_d160(const BwdLaunchArgs &a);
int launch_bwd_bf16_d64(const BwdLaunchArgs &a);
int launch_bwd_bf16_d96(const BwdLaunchArgs &a);
int launch_bwd_bf16_d128(const BwdLaunchArgs &a);
int launch_bwd_bf16_d160(const BwdLaunchArgs &a);

}  // namespace tsdpa
