// C-ABI of the tiled SDPA library: argument validation, tile and split heuristics, dispatch.
// See include/tiled_sdpa.h for the contract of every entry point.
#include "tiled_sdpa.h"

#include <cmath>
#include <cstdint>
#include <limits>
#include <mutex>

#include "sdpa_fwd_launch.h"
#include "sdpa_merge_kernel.h"

// Split states of tiled_sdpa_fwd_kvcache_static: device memory that belongs to the library, one copy per
// GPU the code object is loaded on.  In host code this name is only a handle for hipGetSymbolAddress;
// the address kernels and copies use is the one that call returns (static_scratch_ptr below).
static __device__ __align__(256) unsigned char scratch[TSDPA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kVersion = 300;  // 0.3.0

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // per device: address of that device's copy of `scratch`, once looked up
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device, with that device
// current); nullptr if the runtime cannot name it.  Allocates nothing.
void *static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

bool valid_tile(int tm, int tn, int D)
{
    // 256 query rows per workgroup: an addition to the paper's Table 1 grid, built for 64-row K/V tiles only
    if (tm == 256) return tn == 64;
    if (!(tm == 64 || tm == 128) || !(tn == 32 || tn == 64 || tn == 128)) return false;
    // 128-row K/V tiles up to D = 128 (above D = 64 the kernel works through such a tile in two halves, its
    // score accumulators for 128 rows not fitting the registers beside the output accumulator); at D = 160
    // the four tile slots would take 256 KiB of LDS
    return tn != 128 || D <= 128;
}

// Shape heuristic (the static counterpart of the paper's shape-aware schedule policy, Section 5.6).
void pick_tile(int BH, int S, int D, bool causal, int *tm, int *tn)
{
    // From the tile sweeps on MI355X (every tile of a shape timed in turn, the order reversing from round to
    // round): among the paper's query tiles, 128 rows per workgroup (four wavefronts) win wherever a sequence is
    // longer than two such tiles.  Up to D = 128 the two K/V tile heights are within 2 % of each other on
    // long sequences: 32 rows fit three wavefronts per SIMD, 64 rows halve the barriers and are built
    // with the scheduler that suits them.  The 64-row tile is ahead by 4-14 % on mid-length sequences
    // (512-2048) and under the causal mask, where the finer diagonal of the 32-row tile does not pay
    // for its barriers; at D = 128 its masked step also spills, so every S above one tile takes 64
    // rows there.  Short sequences (S = 197, 333) are level or better on 32 rows at D = 64, 96 and 160.
    // At D = 160 the 64-row tile, whose four slots of unpadded rows are 80 KiB and leave room for two workgroups
    // per CU, is 3-5 % ahead under the mask and 5-20 % ahead without it from S = 512 up to where the 256-row
    // tile below takes over.
    *tm = S <= 64 ? 64 : 128;
    *tn = 32;
    if (D == 128 && S > 64) *tn = 64;
    if (D != 128 && S >= 512) *tn = 64;
    // up to two 128-row tiles per head and fewer of them than CUs: 64 query rows per workgroup start twice as
    // many (1-4 % at D = 128, 2-12 % at D = 160; level at D = 64 and 96)
    if (D >= 128 && S <= 256 && (long long)BH * ((S + 127) / 128) < 256) *tm = 64;
    // many short heads under the mask at D = 96 and 160 (S = 512, 1024; four 128-row workgroups per CU and more):
    // the 64 x 32 tile, which cuts the diagonal finest, is 4-7 % ahead
    if (causal && (D == 96 || D == 160) && S >= 512 && S <= 1024 && (long long)BH * ((S + 127) / 128) >= 1024) {
        *tm = 64;
        *tn = 32;
    }
    // 256 query rows per workgroup (eight wavefronts share every K/V tile: half the tile loads per MFMA; one
    // workgroup per CU) win from D = 96 upward once they give every CU a workgroup and the sequence is long
    // enough: 2-3 % at D = 96 from S = 4096 (level at 2048, 6 % behind there with 256 heads), 3 % at D = 128
    // from S = 2048, 1-2.5 % over 128 x 64 at D = 160 from S = 1024.
    // Not under the causal mask (a workgroup's diagonal band is four masked tiles instead of two and the query
    // tiles of a head balance worse: within 2 % either way at S = 8192 and 16384, 5-25 % slower at S = 2048),
    // not at D = 64 (3-14 % slower).
    const long long wg256 = (long long)BH * ((S + 255) / 256);
    bool wide = !causal && D >= 96 && wg256 >= 256 && S >= (D == 160 ? 1024 : D == 96 ? 4096 : 2048);
    // (D = 160 below S = 4096: ahead while a CU gets up to three such workgroups, 3-4 % behind 128 x 64 with more)
    if (D == 160 && S < 4096 && wg256 >= 1024) wide = false;
    if (wide) {
        *tm = 256;
        *tn = 64;
    }
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

// Splits along the key axis (from timings on MI355X).  None when the query tiles alone give every CU
// two workgroups.  Otherwise aim for two workgroups per CU if every split then still streams 16 tiles
// or more (long caches: more loads in flight pay), else for one per CU, never cutting runs shorter
// than 4 tiles for up to 64 query rows or 16 tiles beyond (each split of a query tile writes and the
// merge re-reads T_M x D floats, which a short run does not amortise).
int pick_splits(int BH, int Sq, int Skv, int tm, int tn)
{
    const int64_t base = (int64_t)BH * ((Sq + tm - 1) / tm);
    const int64_t tiles = (Skv + tn - 1) / tn;
    if (base <= 0 || base >= 512) return 1;
    int64_t want = (512 + base - 1) / base;
    if (tiles / want < 16) {
        want = (256 + base - 1) / base;
        const int64_t shortest = Sq <= 64 ? 4 : 16;
        const int64_t most = tiles / shortest > 1 ? tiles / shortest : 1;
        if (want > most) want = most;
    }
    if (want > TSDPA_MAX_SPLITS) want = TSDPA_MAX_SPLITS;
    return (int)want;
}

int validate_shape_kv(int B, int H, int Sq, int Skv, int D, int dtype, unsigned flags)
{
    if (dtype != TSDPA_F16 && dtype != TSDPA_BF16) return TSDPA_ERR_BAD_DTYPE;
    if (D != 64 && D != 96 && D != 128 && D != 160) return TSDPA_ERR_UNSUPPORTED_D;
    if (B < 0 || H < 0 || Sq < 0 || Skv < 0) return TSDPA_ERR_BAD_SHAPE;
    const int64_t bh = (int64_t)B * (int64_t)H;
    // B*H*ceil(Sq/64)*splits workgroups must fit an int
    if (bh > 0 && Sq > 0 &&
        bh * (((int64_t)Sq + 63) / 64) * TSDPA_MAX_SPLITS > (int64_t)std::numeric_limits<int>::max())
        return TSDPA_ERR_BAD_SHAPE;
    if (((int64_t)Skv + 1024) * D * 2 >= ((int64_t)1 << 30)) return TSDPA_ERR_BAD_SHAPE;
    if (bh > 0 && Sq > 0 && Skv == 0) return TSDPA_ERR_BAD_SHAPE;
    if ((flags & TSDPA_FLAG_CAUSAL) && Skv < Sq) return TSDPA_ERR_BAD_SHAPE;
    return TSDPA_OK;
}

// tiles of the Sq x Skv entry points: T_M in {64,128} x T_N in {32,64}, and 256 x 64 on a dense cache
bool valid_tile_kv(int tm, int tn, bool paged)
{
    if (tm == 256) return tn == 64 && !paged;
    return (tm == 64 || tm == 128) && (tn == 32 || tn == 64);
}

void pick_tile_kv(long long heads, int Sq, int Skv, int D, int *tm, int *tn)
{
    // (decoding shapes are bound by the cache read, not by the loop)
    *tm = Sq <= 64 ? 64 : 128;
    *tn = Skv >= 512 ? 64 : 32;
    // D = 160: 32-row tiles are level or ahead (3-10 %) until the query block is long (2048 rows: 64-row tiles
    // 2-5 % ahead) or its 128-row tiles are fewer than the CUs (15 % ahead at one head's 512 or 1024 rows);
    // D = 96: a handful of query rows per key/value head read the cache 2-15 % faster in 32-row tiles
    if (D == 160) *tn = (Sq >= 2048 || (Sq >= 128 && Skv >= 512 && heads * ((Sq + 127) / 128) < 256)) ? 64 : 32;
    if (D == 96 && Sq <= 16) *tn = 32;
}

}  // namespace

static int fwd_kv_impl(const void *q, const void *k, const void *v, void *o, float *lse, const int *kv_lens,
                       const int *block_table, int max_blocks, int block_shift,
                       int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                       int tile_m, int tile_n, unsigned flags,
                       int splits, void *workspace, unsigned long long workspace_bytes);

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
        case TSDPA_ERR_BAD_TILE: return "bad tile: tile_m in {64,128}, tile_n in {32,64,128} (128 not at D = 160), or (256,64), or both 0";
        case TSDPA_ERR_BAD_SCALE: return "bad scale: must be finite (NaN selects 1/sqrt(D))";
        case TSDPA_ERR_LAUNCH: return "kernel launch failed";
        case TSDPA_ERR_WORKSPACE: return "split workspace is null, misaligned or too small";
        case TSDPA_ERR_BAD_SPLITS: return "bad splits: must be 0 (heuristic) or 1..128";
        case TSDPA_ERR_STATIC_SCRATCH:
            return "split states exceed the library's static scratch buffer (or its address is unavailable): "
                   "use tiled_sdpa_fwd_kvcache with a workspace of the caller's, or fewer splits";
        default: return "unknown status";
    }
}

int tiled_sdpa_default_tile(int B, int H, int S, int D, int dtype, unsigned flags, int *tile_m, int *tile_n)
{
    if (!tile_m || !tile_n) return TSDPA_ERR_NULL_PTR;
    const int st = validate_shape(B, H, S, D, dtype);
    if (st != TSDPA_OK) return st;
    pick_tile(B * H, S, D, (flags & TSDPA_FLAG_CAUSAL) != 0, tile_m, tile_n);
    return TSDPA_OK;
}

int tiled_sdpa_tune_tile(const void *q, const void *k, const void *v, void *o,
                         int B, int H, int S, int D, float scale, int dtype, void *stream, unsigned flags,
                         int launches, int *tile_m, int *tile_n, float *ms_per_launch)
{
    if (!tile_m || !tile_n) return TSDPA_ERR_NULL_PTR;
    if (launches < 1 || launches > 1000) return TSDPA_ERR_BAD_SHAPE;
    int st = validate_shape(B, H, S, D, dtype);
    if (st != TSDPA_OK) return st;
    pick_tile(B * H, S, D, (flags & TSDPA_FLAG_CAUSAL) != 0, tile_m, tile_n);
    if (ms_per_launch)
        for (int i = 0; i < TSDPA_TUNE_TILES; ++i) ms_per_launch[i] = -1.0f;
    if ((int64_t)B * H * S == 0) return TSDPA_OK;
    if (!q || !k || !v || !o) return TSDPA_ERR_NULL_PTR;
    if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15u) != 0) return TSDPA_ERR_MISALIGNED;
    if (std::isinf(scale)) return TSDPA_ERR_BAD_SCALE;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TSDPA_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return TSDPA_ERR_LAUNCH; }
    static const int tms[TSDPA_TUNE_TILES] = {64, 64, 64, 128, 128, 128, 256};
    static const int tns[TSDPA_TUNE_TILES] = {32, 64, 128, 32, 64, 128, 64};
    float best = -1.0f;
    st = TSDPA_OK;
    for (int i = 0; i < TSDPA_TUNE_TILES && st == TSDPA_OK; ++i) {
        const int tm = tms[i], tn = tns[i];
        if (!valid_tile(tm, tn, D)) continue;
        // one untimed launch (first use of an instantiation sets its attributes), then the timed run
        st = tiled_sdpa_fwd_ex(q, k, v, o, nullptr, B, H, S, D, scale, dtype, stream, tm, tn, flags);
        if (st != TSDPA_OK) break;
        if (hipEventRecord(e0, (hipStream_t)stream) != hipSuccess) { st = TSDPA_ERR_LAUNCH; break; }
        for (int r = 0; r < launches && st == TSDPA_OK; ++r)
            st = tiled_sdpa_fwd_ex(q, k, v, o, nullptr, B, H, S, D, scale, dtype, stream, tm, tn, flags);
        if (st != TSDPA_OK) break;
        float ms = 0.0f;
        if (hipEventRecord(e1, (hipStream_t)stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { st = TSDPA_ERR_LAUNCH; break; }
        ms /= (float)launches;
        if (ms_per_launch) ms_per_launch[i] = ms;
        if (best < 0.0f || ms < best) { best = ms; *tile_m = tm; *tile_n = tn; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
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
        pick_tile(B * H, S, D, (flags & TSDPA_FLAG_CAUSAL) != 0, &tile_m, &tile_n);
    else if (!valid_tile(tile_m, tile_n, D))
        return TSDPA_ERR_BAD_TILE;
    if (std::isnan(scale)) scale = 1.0f / std::sqrt((float)D);
    if (std::isinf(scale)) return TSDPA_ERR_BAD_SCALE;

    tsdpa::LaunchArgs a{};
    a.q = q;
    a.k = k;
    a.v = v;
    a.o = o;
    a.lse = lse;
    a.BH = B * H;
    a.S = S;
    a.rows_per_head = S;
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

unsigned long long tiled_sdpa_kv_workspace_bytes(int B, int H, int Sq, int D, int splits)
{
    if (B < 0 || H < 0 || Sq < 0 || D < 0 || splits <= 1) return 0;
    return (unsigned long long)B * H * splits * Sq * (D + 2) * sizeof(float);
}

int tiled_sdpa_kv_default_splits(int B, int H, int Sq, int Skv, int D, int dtype, unsigned flags, int *splits)
{
    if (!splits) return TSDPA_ERR_NULL_PTR;
    const int st = validate_shape_kv(B, H, Sq, Skv, D, dtype, flags);
    if (st != TSDPA_OK) return st;
    int tm, tn;
    pick_tile_kv((long long)B * H, Sq, Skv, D, &tm, &tn);
    *splits = pick_splits(B * H, Sq, Skv, tm, tn);
    return TSDPA_OK;
}

int tiled_sdpa_fwd_kv(const void *q, const void *k, const void *v, void *o, float *lse,
                      int B, int H, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                      int tile_m, int tile_n, unsigned flags,
                      int splits, void *workspace, unsigned long long workspace_bytes)
{
    return tiled_sdpa_fwd_gqa(q, k, v, o, lse, B, H, H, Sq, Skv, D, scale, dtype, stream, tile_m, tile_n, flags,
                              splits, workspace, workspace_bytes);
}

int tiled_sdpa_fwd_gqa(const void *q, const void *k, const void *v, void *o, float *lse,
                       int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                       int tile_m, int tile_n, unsigned flags,
                       int splits, void *workspace, unsigned long long workspace_bytes)
{
    return tiled_sdpa_fwd_kvcache(q, k, v, o, lse, nullptr, B, H, Hkv, Sq, Skv, D, scale, dtype, stream, tile_m,
                                  tile_n, flags, splits, workspace, workspace_bytes);
}

int tiled_sdpa_fwd_kvcache(const void *q, const void *k, const void *v, void *o, float *lse, const int *kv_lens,
                           int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                           int tile_m, int tile_n, unsigned flags,
                           int splits, void *workspace, unsigned long long workspace_bytes)
{
    return fwd_kv_impl(q, k, v, o, lse, kv_lens, nullptr, 0, 0, B, H, Hkv, Sq, Skv, D, scale, dtype, stream, tile_m,
                       tile_n, flags, splits, workspace, workspace_bytes);
}

int tiled_sdpa_fwd_kvcache_static(const void *q, const void *k, const void *v, void *o, float *lse,
                                  const int *kv_lens, int B, int H, int Hkv, int Sq, int Skv, int D, float scale,
                                  int dtype, void *stream, int tile_m, int tile_n, unsigned flags, int splits)
{
    // the checks that decide the split count, in the order of tiled_sdpa_fwd_kvcache, so that the size
    // of the split states is known before anything is enqueued
    int st = validate_shape_kv(B, H, Sq, Skv, D, dtype, flags);
    if (st != TSDPA_OK) return st;
    if (Hkv < 0 || (H > 0 && (Hkv == 0 || H % Hkv != 0))) return TSDPA_ERR_BAD_SHAPE;
    if ((int64_t)B * H * Sq == 0) return TSDPA_OK;
    if (splits < 0 || splits > TSDPA_MAX_SPLITS) return TSDPA_ERR_BAD_SPLITS;
    if ((int64_t)(H / Hkv) * Sq > (int64_t)std::numeric_limits<int>::max()) return TSDPA_ERR_BAD_SHAPE;
    if (splits == 0) {
        int tm = tile_m, tn = tile_n;
        if (tm == 0 && tn == 0) pick_tile_kv((long long)B * Hkv, (H / Hkv) * Sq, Skv, D, &tm, &tn);
        else if (!valid_tile_kv(tm, tn, false)) return TSDPA_ERR_BAD_TILE;
        splits = pick_splits(B * Hkv, (H / Hkv) * Sq, Skv, tm, tn);
    }
    const unsigned long long need = tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, splits);
    if (need > (unsigned long long)TSDPA_STATIC_SCRATCH_BYTES) return TSDPA_ERR_STATIC_SCRATCH;
    void *ws = nullptr;
    if (need > 0) {
        ws = static_scratch_ptr();
        if (ws == nullptr) return TSDPA_ERR_STATIC_SCRATCH;
    }
    // every word of the split states that the merge kernel reads is written by the attention kernel of
    // the same call (a split without tiles stores (0, -inf, 0)), so nothing has to be cleared
    return fwd_kv_impl(q, k, v, o, lse, kv_lens, nullptr, 0, 0, B, H, Hkv, Sq, Skv, D, scale, dtype, stream, tile_m,
                       tile_n, flags, splits, ws, need);
}

int tiled_sdpa_fwd_paged(const void *q, const void *k_pages, const void *v_pages, void *o, float *lse,
                         const int *kv_lens, const int *block_table,
                         int B, int H, int Hkv, int Sq, int max_blocks, int block_rows, int D,
                         float scale, int dtype, void *stream, int tile_m, int tile_n, unsigned flags,
                         int splits, void *workspace, unsigned long long workspace_bytes)
{
    // pages of 64 << n rows, so that a K/V tile of 32 or 64 rows never straddles two pages
    int shift = 6;
    while (shift < 20 && (1 << shift) != block_rows) ++shift;
    if (max_blocks < 0 || (1 << shift) != block_rows) return TSDPA_ERR_BAD_SHAPE;
    if ((int64_t)max_blocks * block_rows > (int64_t)std::numeric_limits<int>::max()) return TSDPA_ERR_BAD_SHAPE;
    const int cap = max_blocks * block_rows;
    const int st = validate_shape_kv(B, H, Sq, cap, D, dtype, flags);
    if (st != TSDPA_OK) return st;
    if ((int64_t)B * H * Sq != 0 && (!kv_lens || !block_table)) return TSDPA_ERR_NULL_PTR;
    if (((uintptr_t)block_table & 3u) != 0) return TSDPA_ERR_MISALIGNED;
    return fwd_kv_impl(q, k_pages, v_pages, o, lse, kv_lens, block_table, max_blocks, shift, B, H, Hkv, Sq, cap, D,
                       scale, dtype, stream, tile_m, tile_n, flags, splits, workspace, workspace_bytes);
}

}  // extern "C"

// Everything behind tiled_sdpa_fwd_kv / _gqa / _kvcache / _paged: one query block per query head against a
// cache of Skv rows per key/value head, dense (block_table NULL) or paged.
static int fwd_kv_impl(const void *q, const void *k, const void *v, void *o, float *lse, const int *kv_lens,
                       const int *block_table, int max_blocks, int block_shift,
                       int B, int H, int Hkv, int Sq, int Skv, int D, float scale, int dtype, void *stream,
                       int tile_m, int tile_n, unsigned flags,
                       int splits, void *workspace, unsigned long long workspace_bytes)
{
    int st = validate_shape_kv(B, H, Sq, Skv, D, dtype, flags);
    if (st != TSDPA_OK) return st;
    if (Hkv < 0 || (H > 0 && (Hkv == 0 || H % Hkv != 0))) return TSDPA_ERR_BAD_SHAPE;
    if ((int64_t)B * H * Sq == 0) return TSDPA_OK;
    // the G query heads of a group are adjacent, so q, o and lse are also [B, Hkv, G*Sq, ...]: the
    // kernel runs one "head" per key/value head over the G*Sq rows that read it
    const int G = H / Hkv;
    if ((int64_t)G * Sq > (int64_t)std::numeric_limits<int>::max()) return TSDPA_ERR_BAD_SHAPE;
    const int rows = G * Sq;
    if (!q || !k || !v || !o) return TSDPA_ERR_NULL_PTR;
    const uintptr_t bits = (uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o;
    if ((bits & 15u) != 0 || (((uintptr_t)lse | (uintptr_t)kv_lens) & 3u) != 0) return TSDPA_ERR_MISALIGNED;
    const bool heuristic_tile = tile_m == 0 && tile_n == 0;
    if (heuristic_tile)
        pick_tile_kv((long long)B * Hkv, rows, Skv, D, &tile_m, &tile_n);
    else if (!valid_tile_kv(tile_m, tile_n, block_table != nullptr))
        return TSDPA_ERR_BAD_TILE;
    if (std::isnan(scale)) scale = 1.0f / std::sqrt((float)D);
    if (std::isinf(scale)) return TSDPA_ERR_BAD_SCALE;
    if (splits < 0 || splits > TSDPA_MAX_SPLITS) return TSDPA_ERR_BAD_SPLITS;
    if (splits == 0) splits = pick_splits(B * Hkv, rows, Skv, tile_m, tile_n);
    // Long query blocks against a dense cache of one length, no mask, no split: the 256-row query tile of the
    // square problem, under the same conditions (with 256 such workgroups the 128-row tile has 512 and is not
    // split either, so the split count does not depend on this choice)
    if (heuristic_tile && splits == 1 && block_table == nullptr && kv_lens == nullptr &&
        !(flags & TSDPA_FLAG_CAUSAL) && D >= 96 && rows >= (D == 160 ? 1024 : D == 96 ? 4096 : 2048) &&
        (int64_t)B * Hkv * ((rows + 255) / 256) >= 256) {
        tile_m = 256;
        tile_n = 64;
    }
    if (splits > 1) {
        if (!workspace || ((uintptr_t)workspace & 15u) != 0 ||
            workspace_bytes < tiled_sdpa_kv_workspace_bytes(B, H, Sq, D, splits))
            return TSDPA_ERR_WORKSPACE;
    }

    tsdpa::LaunchArgs a{};
    a.q = q;
    a.k = k;
    a.v = v;
    a.o = o;
    a.lse = lse;
    a.BH = B * Hkv;
    a.S = rows;
    a.rows_per_head = Sq;
    a.kv_lens = kv_lens;
    a.heads_per_batch = Hkv;
    a.block_table = block_table;
    a.max_blocks = max_blocks;
    a.block_shift = block_shift;
    a.tile_rot = (block_table == nullptr && rows <= tile_m) ? 1 : 0;    // one query tile per head: see the kernel
    a.c = std::fabs(scale) * 1.44269504088896340736f;
    a.tau = (flags & TSDPA_FLAG_EXACT_MAX) ? 0.0f : 8.0f;
    a.qsign = std::signbit(scale) && scale != 0.0f ? 0x80008000u : 0u;
    a.linear_grid = (flags & TSDPA_FLAG_LINEAR_GRID) ? 1 : 0;
    a.causal = (flags & TSDPA_FLAG_CAUSAL) ? 1 : 0;
    a.kv = 1;
    a.Skv = Skv;
    a.splits = splits;
    a.ws = (float *)workspace;
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
    if (err != 0) return TSDPA_ERR_LAUNCH;
    const size_t out_rows = (size_t)B * H * Sq;
    // Which merge: with more than eight splits a thread that walks them waits for its loads in several
    // batches, and when the rows are few (decoding) nothing else hides that: one workgroup per row, the
    // splits shared among eight threads (32 splits of 32 rows: 3.5 us against 12.5 us).  With thousands of
    // rows the walking threads are many enough to hide it themselves and launch an eighth of the threads
    // (8 splits of 8192 rows: 47 us per call against 55 us).
    if (splits > 8 && out_rows <= 2048) {
        static_assert(tsdpa::kMergeLanes * tsdpa::kMergePerLane >= TSDPA_MAX_SPLITS, "every split needs a thread");
        const dim3 block(D / 4, tsdpa::kMergeLanes);
        if (dtype == TSDPA_F16)
            hipLaunchKernelGGL(tsdpa::sdpa_merge_wide_kernel<_Float16>, dim3((unsigned)out_rows), block, 0, (hipStream_t)stream,
                               (const float *)workspace, (_Float16 *)o, lse, B * Hkv, rows, D, splits);
        else
            hipLaunchKernelGGL(tsdpa::sdpa_merge_wide_kernel<__bf16>, dim3((unsigned)out_rows), block, 0, (hipStream_t)stream,
                               (const float *)workspace, (__bf16 *)o, lse, B * Hkv, rows, D, splits);
        if (hipGetLastError() != hipSuccess) return TSDPA_ERR_LAUNCH;
    } else if (splits > 1) {
        const size_t threads = out_rows * (D / 4);
        const unsigned blocks = (unsigned)((threads + 255) / 256);
        if (dtype == TSDPA_F16)
            hipLaunchKernelGGL(tsdpa::sdpa_merge_kernel<_Float16>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                               (const float *)workspace, (_Float16 *)o, lse, B * Hkv, rows, D, splits);
        else
            hipLaunchKernelGGL(tsdpa::sdpa_merge_kernel<__bf16>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                               (const float *)workspace, (__bf16 *)o, lse, B * Hkv, rows, D, splits);
        if (hipGetLastError() != hipSuccess) return TSDPA_ERR_LAUNCH;
    }
    return TSDPA_OK;
}

extern "C" {

unsigned long long tiled_sdpa_bwd_workspace_bytes(int B, int H, int S)
{
    if (B < 0 || H < 0 || S < 0) return 0;
    return 2ull * ((unsigned long long)B * H * S + tsdpa::kBwdStatPad) * sizeof(float);
}

int tiled_sdpa_bwd(const void *q, const void *k, const void *v, const void *o, const void *dout,
                   const float *lse, void *dq, void *dk, void *dv,
                   int B, int H, int S, int D, float scale, int dtype, unsigned flags,
                   void *workspace, unsigned long long workspace_bytes, void *stream)
{
    return tiled_sdpa_bwd_gqa(q, k, v, o, dout, lse, dq, dk, dv, B, H, H, S, D, scale, dtype, flags, workspace,
                              workspace_bytes, stream);
}

int tiled_sdpa_bwd_gqa(const void *q, const void *k, const void *v, const void *o, const void *dout,
                       const float *lse, void *dq, void *dk, void *dv,
                       int B, int H, int Hkv, int S, int D, float scale, int dtype, unsigned flags,
                       void *workspace, unsigned long long workspace_bytes, void *stream)
{
    if (dtype != TSDPA_F16 && dtype != TSDPA_BF16) return TSDPA_ERR_BAD_DTYPE;
    int st = validate_shape(B, H, S, D, dtype);
    if (st != TSDPA_OK) return st;
    if (Hkv < 0 || (H > 0 && (Hkv == 0 || H % Hkv != 0))) return TSDPA_ERR_BAD_SHAPE;
    // the statistics arrays are addressed through a 32-bit byte range
    if ((int64_t)B * H * S >= ((int64_t)1 << 29)) return TSDPA_ERR_BAD_SHAPE;
    if ((int64_t)B * H * S == 0) return TSDPA_OK;
    if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv) return TSDPA_ERR_NULL_PTR;
    const uintptr_t bits = (uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)dout |
                           (uintptr_t)dq | (uintptr_t)dk | (uintptr_t)dv;
    if ((bits & 15u) != 0 || ((uintptr_t)lse & 3u) != 0) return TSDPA_ERR_MISALIGNED;
    if (std::isnan(scale)) scale = 1.0f / std::sqrt((float)D);
    if (std::isinf(scale)) return TSDPA_ERR_BAD_SCALE;
    if (!workspace || ((uintptr_t)workspace & 15u) != 0 ||
        workspace_bytes < tiled_sdpa_bwd_workspace_bytes(B, H, S))
        return TSDPA_ERR_WORKSPACE;

    tsdpa::BwdLaunchArgs a{};
    a.q = q; a.k = k; a.v = v; a.o = o; a.dout = dout; a.lse = lse;
    a.dq = dq; a.dk = dk; a.dv = dv;
    const size_t half = (size_t)B * H * S + tsdpa::kBwdStatPad;
    a.delta = (float *)workspace;
    a.lse2 = (float *)workspace + half;
    a.stat_bytes = (unsigned)(half * sizeof(float));
    a.BH = B * H;
    a.S = S;
    a.group = H / Hkv;
    a.c = std::fabs(scale) * 1.44269504088896340736f;
    a.scale = scale;
    a.rsign = std::signbit(scale) && scale != 0.0f ? 0x80008000u : 0u;
    a.causal = (flags & TSDPA_FLAG_CAUSAL) ? 1 : 0;
    a.stream = (hipStream_t)stream;
    int err;
    if (dtype == TSDPA_F16) {
        switch (D) {
            case 64: err = tsdpa::launch_bwd_f16_d64(a); break;
            case 96: err = tsdpa::launch_bwd_f16_d96(a); break;
            case 128: err = tsdpa::launch_bwd_f16_d128(a); break;
            default: err = tsdpa::launch_bwd_f16_d160(a); break;
        }
    } else {
        switch (D) {
            case 64: err = tsdpa::launch_bwd_bf16_d64(a); break;
            case 96: err = tsdpa::launch_bwd_bf16_d96(a); break;
            case 128: err = tsdpa::launch_bwd_bf16_d128(a); break;
            default: err = tsdpa::launch_bwd_bf16_d160(a); break;
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
