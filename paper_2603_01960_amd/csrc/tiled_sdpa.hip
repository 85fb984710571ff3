// C-ABI of the tiled SDPA forward library: argument validation, tile heuristic, dispatch.
// See include/tiled_sdpa.h for the contract of every entry point.
#include "tiled_sdpa.h"

#include <cmath>
#include <cstdint>
#include <limits>

#include "sdpa_fwd_launch.h"

namespace {

constexpr int kVersion = 100;  // 0.1.0

bool valid_tile(int tm, int tn, int D)
{
    if (!(tm == 64 || tm == 128) || !(tn == 32 || tn == 64 || tn == 128)) return false;
    return !(D == 160 && tn == 128);   // four 128 x 512-byte tiles do not fit the 160 KB LDS
}

// Shape heuristic (the static counterpart of the paper's shape-aware schedule policy, Section 5.6).
void pick_tile(int BH, int S, int D, int *tm, int *tn)
{
    (void)BH;
        // From the tile sweeps on MI355X: 128 query rows per workgroup (four wavefronts, two workgroups per
    // CU) wins at every configuration measured; 64-row K/V tiles for long sequences, 32-row tiles when
    // there are only a few tiles per head, so the pipeline fills sooner and the ragged tail wastes less.
    *tm = 128;
    *tn = S >= 512 ? 64 : 32;
    if (D == 160) *tn = 32;       // 512-byte LDS rows: keeps two workgroups per CU
    if (S <= 64) *tm = 64;
}

int validate_shape(int B, int H, int S, int D, int dtype)
{
    if (dtype != TSDPA_F16 && dtype != TSDPA_BF16) return TSDPA_ERR_BAD_DTYPE;
    if (D != 64 && D != 96 && D != 128 && D != 160) return TSDPA_ERR_UNSUPPORTED_D;
    if (B < 0 || H < 0 || S < 0) return TSDPA_ERR_BAD_SHAPE;
    const int64_t bh = (int64_t)B * (int64_t)H;
    // the grid is B*H*ceil(S/tile_m) <= B*H*ceil(S/64) workgroups and must fit an int
    if (bh > 0 && S > 0 && bh * (((int64_t)S + 63) / 64) > (int64_t)std::numeric_limits<int>::max())
        return TSDPA_ERR_BAD_SHAPE;
    // one head's K (or V) is addressed through a 32-bit byte range with room for a "fetch nothing"
    // offset above it: keep it, prefetch distance included, below 2^30 bytes
    if (((int64_t)S + 1024) * D * 2 >= ((int64_t)1 << 30)) return TSDPA_ERR_BAD_SHAPE;
    return TSDPA_OK;
}

}  // namespace

extern "C" {

int tiled_sdpa_version(void) { return kVersion; }

const char *tiled_sdpa_status_string(int status)
{
    switch (status) {
        case TSDPA_OK: return "ok";
        case TSDPA_ERR_NULL_PTR: return "null pointer for q, k, v or o";
        case TSDPA_ERR_BAD_SHAPE: return "bad shape: B, H, S must be >= 0 and the grid must fit an int";
        case TSDPA_ERR_BAD_DTYPE: return "bad dtype: expected TSDPA_F16 or TSDPA_BF16";
        case TSDPA_ERR_UNSUPPORTED_D: return "unsupported head dimension: D must be 64, 96, 128 or 160";
        case TSDPA_ERR_MISALIGNED: return "misaligned pointer: q, k, v, o need 16-byte, lse 4-byte alignment";
        case TSDPA_ERR_BAD_TILE: return "bad tile: tile_m in {64,128}, tile_n in {32,64,128}, or both 0";
        case TSDPA_ERR_BAD_SCALE: return "bad scale: must be finite (NaN selects 1/sqrt(D))";
        case TSDPA_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int tiled_sdpa_default_tile(int B, int H, int S, int D, int dtype, int *tile_m, int *tile_n)
{
    if (!tile_m || !tile_n) return TSDPA_ERR_NULL_PTR;
    const int st = validate_shape(B, H, S, D, dtype);
    if (st != TSDPA_OK) return st;
    pick_tile(B * H, S, D, tile_m, tile_n);
    return TSDPA_OK;
}

int tiled_sdpa_fwd_ex(const void *q, const void *k, const void *v, void *o, float *lse,
                      int B, int H, int S, int D, float scale, int dtype, void *stream,
                      int tile_m, int tile_n, unsigned flags)
{
    int st = validate_shape(B, H, S, D, dtype);
    if (st != TSDPA_OK) return st;
    if ((int64_t)B * H * S == 0) return TSDPA_OK;
    if (!q || !k || !v || !o) return TSDPA_ERR_NULL_PTR;
    const uintptr_t bits = (uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o;
    if ((bits & 15u) != 0 || ((uintptr_t)lse & 3u) != 0) return TSDPA_ERR_MISALIGNED;
    if (tile_m == 0 && tile_n == 0)
        pick_tile(B * H, S, D, &tile_m, &tile_n);
    else if (!valid_tile(tile_m, tile_n, D))
        return TSDPA_ERR_BAD_TILE;
    if (std::isnan(scale)) scale = 1.0f / std::sqrt((float)D);
    if (std::isinf(scale)) return TSDPA_ERR_BAD_SCALE;

    tsdpa::LaunchArgs a;
    a.q = q;
    a.k = k;
    a.v = v;
    a.o = o;
    a.lse = lse;
    a.BH = B * H;
    a.S = S;
    a.c = std::fabs(scale) * 1.44269504088896340736f;
    a.tau = (flags & TSDPA_FLAG_EXACT_MAX) ? 0.0f : 8.0f;
    a.qsign = std::signbit(scale) && scale != 0.0f ? 0x80008000u : 0u;
    a.linear_grid = (flags & TSDPA_FLAG_LINEAR_GRID) ? 1 : 0;
    a.causal = (flags & TSDPA_FLAG_CAUSAL) ? 1 : 0;
    a.stream = (hipStream_t)stream;

    int err;
    if (dtype == TSDPA_F16) {
        switch (D) {
            case 64: err = tsdpa::launch_f16_d64(tile_m, tile_n, a); break;
            case 96: err = tsdpa::launch_f16_d96(tile_m, tile_n, a); break;
            case 128: err = tsdpa::launch_f16_d128(tile_m, tile_n, a); break;
            default: err = tsdpa::launch_f16_d160(tile_m, tile_n, a); break;
        }
    } else {
        switch (D) {
            case 64: err = tsdpa::launch_bf16_d64(tile_m, tile_n, a); break;
            case 96: err = tsdpa::launch_bf16_d96(tile_m, tile_n, a); break;
            case 128: err = tsdpa::launch_bf16_d128(tile_m, tile_n, a); break;
            default: err = tsdpa::launch_bf16_d160(tile_m, tile_n, a); break;
        }
    }
    return err == 0 ? TSDPA_OK : TSDPA_ERR_LAUNCH;
}

int tiled_sdpa_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
                   int B, int H, int S, int D, float scale, int dtype, void *stream)
{
    return tiled_sdpa_fwd_ex(q, k, v, o, lse, B, H, S, D, scale, dtype, stream, 0, 0, 0u);
}

}  // extern "C"
